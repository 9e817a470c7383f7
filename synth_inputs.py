"""Seeded synthetic inputs for the HIPPO hot path (video-shaped KV caches).

This module only *draws data*.  It holds none of the method's arithmetic (no
softmax, no cosine similarity, no normalisation of scores, no selection): it is
the one module both the CPU oracle's tests and the HIP path's tests/bench may
import.  Everything is produced by ``numpy.random.default_rng(seed)``.

The inputs stand in for the paper's workloads (long videos run through
video-LLMs; 64 or 128 frames of ~196 tokens each plus a text prompt, App.
"Details of Experimental Setups"): only shapes and coarse statistics are
imitated.

Sequence layout of a cache (per batch element, per KV head)::

    [ n_prefix text | F frames, each grid_h x grid_w row-major | n_suffix text | q_len new rows ]

so ``ctx_len = n_prefix + N_v + n_suffix`` and the cache holds ``ctx_len + q_len``
rows.  Arrays are float32 whose values are exactly representable in the config's
dtype (bf16 configs are rounded to bf16, round-to-nearest-even, before anyone
sees them), so the oracle and the GPU read bit-identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    dtype: str          # "fp32" | "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_frames: int
    grid_h: int
    grid_w: int
    n_prefix: int       # text tokens before the video
    n_suffix: int       # text tokens after the video (these are the text queries)
    gamma: int          # draft tokens per round; verify q_len = gamma + 1
    keep_pct: int       # percent of visual tokens kept
    q_unscaled: bool    # True: query entries ~ N(0,1); False: N(0,1)/sqrt(d)
    crop_h: int = 5
    crop_w: int = 5

    @property
    def n_visual(self) -> int:
        return self.n_frames * self.grid_h * self.grid_w

    @property
    def ctx_len(self) -> int:
        return self.n_prefix + self.n_visual + self.n_suffix

    @property
    def q_len(self) -> int:
        return self.gamma + 1

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def k_keep(self) -> int:
        # integer ceil(keep_pct% of N_v): 10 % of 768 -> 77
        return (self.n_visual * self.keep_pct + 99) // 100

    @property
    def l_txt(self) -> int:
        return self.n_suffix

    def with_keep(self, pct: int) -> "Config":
        return replace(self, keep_pct=pct)


CONFIGS: Dict[str, Config] = {
    # 1 layer, 4 q heads / 2 KV heads, d 64, fp32, 32 + 4x(12x16) + 32 = 832, gamma 4
    "tiny": Config("tiny", "fp32", 1, 4, 2, 64, 4, 12, 16, 32, 32, 4, 10, False),
    # 14 / 2 heads, d 64, bf16, 16 x (16x16) + 128 text, gamma 5
    "draft": Config("draft", "bf16", 1, 14, 2, 64, 16, 16, 16, 64, 64, 5, 10, True),
    # 28 / 4 heads, d 128, bf16, 64 x (16x16) + 256 text, gamma 5  (the 16K headline config)
    "c3_16k": Config("c3_16k", "bf16", 1, 28, 4, 128, 64, 16, 16, 128, 128, 5, 10, True),
    # 28 / 4 heads, d 128, bf16, 128 x (16x16) + 512 text, gamma 8
    "c4_long": Config("c4_long", "bf16", 1, 28, 4, 128, 128, 16, 16, 256, 256, 8, 10, True),
    # 64 / 8 heads, d 128, bf16, batch 4, 64 x (24x24) + 256 text, gamma 5
    "c5_large": Config("c5_large", "bf16", 4, 64, 8, 128, 64, 24, 24, 128, 128, 5, 10, True),
}


# ----------------------------------------------------------------------------------------------
# dtype plumbing (formatting of inputs, not method arithmetic)
# ----------------------------------------------------------------------------------------------

def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array holding the nearest bf16 values (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array of bf16-representable values -> uint16 array of bf16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _fmt(cfg: Config, x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    return round_to_bf16(x) if cfg.dtype == "bf16" else x


# ----------------------------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------------------------

def _smooth_field(rng: np.random.Generator, cfg: Config) -> np.ndarray:
    """Per-frame smooth random field for the visual keys of one batch element.

    Returns [H_kv, F, grid_h, grid_w, d].  Channel c of KV head h in frame f is
    sum_{m<4} a_m sin(2 pi (u_m x/W + w_m y/H) + phi_m(f)); amplitudes and
    frequencies are drawn once per (head, channel), the phases random-walk by
    U(-0.5, 0.5) rad per frame so neighbouring frames resemble each other.
    """
    hk, d, F, gh, gw = cfg.n_kv_heads, cfg.head_dim, cfg.n_frames, cfg.grid_h, cfg.grid_w
    a = rng.uniform(0.5, 1.0, size=(hk, d, 4))
    u = rng.uniform(0.0, 2.0, size=(hk, d, 4))
    w = rng.uniform(0.0, 2.0, size=(hk, d, 4))
    phi0 = rng.uniform(0.0, 2.0 * np.pi, size=(hk, d, 4))
    drift = rng.uniform(-0.5, 0.5, size=(F, hk, d, 4))
    drift[0] = 0.0
    phi = phi0[None] + np.cumsum(drift, axis=0)                     # [F,hk,d,4]
    xs = np.arange(gw) / gw
    ys = np.arange(gh) / gh
    ax = 2.0 * np.pi * u[..., None] * xs                            # [hk,d,4,gw]
    by = 2.0 * np.pi * w[..., None] * ys                            # [hk,d,4,gh]
    # sin(ax + by + phi) = sin(ax+phi) cos(by) + cos(ax+phi) sin(by)
    axp = ax[None] + phi[..., None]                                 # [F,hk,d,4,gw]
    sx, cx = np.sin(axp), np.cos(axp)
    sy, cy = np.sin(by), np.cos(by)
    field = np.einsum("hcm,fhcmx,hcmy->hfyxc", a, sx, cy, optimize=True)
    field += np.einsum("hcm,fhcmx,hcmy->hfyxc", a, cx, sy, optimize=True)
    return field.astype(np.float32)


def make_inputs(cfg: Config, seed: int = 0) -> Dict[str, np.ndarray]:
    """All tensors of one layer of one config.

    Keys of the result
      q_txt   [B, L_txt, H, d]        text-prompt queries (suffix text tokens)
      k, v    [B, H_kv, ctx_len+q_len, d]   full cache incl. the q_len appended rows
      q_new   [B, q_len, H, d]        the gamma+1 verify queries (row 0 also serves as a draft query)
    """
    rng = np.random.default_rng(seed)
    B, H, hk, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    F, gh, gw = cfg.n_frames, cfg.grid_h, cfg.grid_w
    G = cfg.group
    n_tot = cfg.ctx_len + cfg.q_len
    inv = 1.0 / np.sqrt(d)
    qs = 1.0 if cfg.q_unscaled else inv

    # text queries: iid normal plus a component shared by the G heads of a KV head, so that a
    # "mean query direction" exists (real prompts' queries share one; it is what attention sinks
    # and the frame-boundary bias latch onto)
    shared = rng.standard_normal((B, hk, d))
    shared /= np.linalg.norm(shared, axis=-1, keepdims=True)
    q_txt = rng.standard_normal((B, cfg.l_txt, H, d))
    q_txt += 0.6 * np.sqrt(d) * np.repeat(shared, G, axis=1)[:, None, :, :]
    q_txt = _fmt(cfg, q_txt * qs)

    q_new = _fmt(cfg, rng.standard_normal((B, cfg.q_len, H, d)) * qs)

    v = rng.standard_normal((B, hk, n_tot, d), dtype=np.float32) * np.float32(inv)
    k = rng.standard_normal((B, hk, n_tot, d), dtype=np.float32) * np.float32(inv)

    ring = np.zeros((gh, gw), dtype=bool)
    ring[0, :] = ring[-1, :] = True
    ring[:, 0] = ring[:, -1] = True
    v0 = cfg.n_prefix
    for b in range(B):
        field = _smooth_field(rng, cfg)                              # [hk,F,gh,gw,d]
        field += np.float32(0.3) * rng.standard_normal(field.shape, dtype=np.float32)
        field *= np.float32(inv)
        # position bias: +1.5 along the mean text-query direction on the outer ring of each frame
        qm = q_txt[b].astype(np.float64).reshape(cfg.l_txt, hk, G, d).mean(axis=(0, 2))  # [hk,d]
        qm /= np.maximum(np.linalg.norm(qm, axis=-1, keepdims=True), 1e-30)
        field[:, :, ring, :] += (1.5 * qm[:, None, None, :]).astype(np.float32)
        k[b, :, v0:v0 + cfg.n_visual, :] = field.reshape(hk, cfg.n_visual, d)

    return {"q_txt": q_txt, "k": _fmt(cfg, k), "v": _fmt(cfg, v), "q_new": q_new}


def random_scores(n_batch: int, n: int, seed: int, n_distinct: int = 0) -> np.ndarray:
    """fp32 score rows for top-k tests; n_distinct > 0 plants many exact ties."""
    rng = np.random.default_rng(seed)
    if n_distinct > 0:
        vals = rng.standard_normal(n_distinct).astype(np.float32)
        return vals[rng.integers(0, n_distinct, size=(n_batch, n))]
    return rng.standard_normal((n_batch, n)).astype(np.float32)


LM_VOCAB = 152064      # rows of the LM head of the 7B-class models the paper evaluates (Qwen2 family)


def make_logits(n_batch: int, gamma: int, vocab: int, seed: int, closeness: float = 0.6):
    """Target logits [B, gamma+1, V] and draft logits [B, gamma, V] for speculative-sampling
    verification: an LM-head-like row (a few likely words far above a long Gaussian tail); the draft's
    row is the target's plus noise of scale `closeness`, so acceptance is neither certain nor hopeless.
    Returns (p_logits, q_logits, rng) -- the generator is handed back for the uniforms."""
    rng = np.random.default_rng(seed)
    pl = rng.standard_normal((n_batch, gamma + 1, vocab)).astype(np.float32) * 2.0
    hot = rng.integers(0, vocab, (n_batch, gamma + 1, 4))
    np.put_along_axis(pl, hot, pl.max() + rng.random((n_batch, gamma + 1, 4)).astype(np.float32) * 4.0, axis=-1)
    ql = pl[:, :gamma] + closeness * rng.standard_normal((n_batch, gamma, vocab)).astype(np.float32)
    return pl, ql, rng


def quantize_e4m3(x: np.ndarray):
    """[B,Hkv,N,d] float array -> (uint8 E4M3 codes of the same shape, fp32 multipliers [B,Hkv]) with
    multiplier = max|x| / 448 per (batch element, KV head) and codes = x / multiplier rounded to the
    nearest representable value (ties to even) by the tensor library's own conversion.  Input
    formatting only, like the bf16 rounding above."""
    import torch
    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=(2, 3))
    mult = np.where(amax > 0, amax / 448.0, 1.0).astype(np.float32)
    y = torch.from_numpy(x / mult[:, :, None, None]).clamp_(-448.0, 448.0)
    codes = y.to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()
    return codes, mult
