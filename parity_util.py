"""Helpers shared by the GPU parity tests, the smoke run and the benchmark: host<->device marshalling
and the tolerances.  No arithmetic of the method lives here.

Tolerances (stated by the benchmark definition, with the reading used for values that cross zero):
  fp32 : |x - ref| <= 1e-5 * max(|ref|, rms(ref))
  bf16 : |x - ref| <= 2e-2 + 2e-2 * |ref|
and, because attention outputs on these inputs are far smaller than 2e-2, a second bound without
the absolute term, derived from the kernel's arithmetic (P rounded to bf16 before the PV product:
relative 2^-9 per term, so up to 2^-9 * sum_n p_n |v_n|, which under cancellation is a few times
2^-9 |out|; output rounded to bf16: relative 2^-9; everything else fp32):
  bf16 : |x - ref| <= 2e-2 * max(|ref|, rms(ref))
"""
import numpy as np
import torch

import synth_inputs as si


def dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        bits = si.bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def prep(x: np.ndarray, dtype: str) -> np.ndarray:
    """values as the GPU will see them (bf16 inputs rounded), float32"""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return si.round_to_bf16(x) if dtype == "bf16" else x


def assert_close(got: np.ndarray, ref: np.ndarray, dtype: str, what: str = ""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    err = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref ** 2)))
    floor = np.maximum(np.abs(ref), rms)
    if dtype == "fp32":
        bad = err > 1e-5 * floor
    else:
        bad = (err > 2e-2 + 2e-2 * np.abs(ref)) | (err > 2e-2 * floor)
    if bad.any():
        i = np.unravel_index(np.argmax(err / np.maximum(floor, 1e-300)), err.shape)
        raise AssertionError("%s: %d of %d outside tolerance; worst at %s got %.9g ref %.9g (rms %.3g)"
                             % (what, int(bad.sum()), bad.size, i, got[i], ref[i], rms))


def assert_fused_close(got: np.ndarray, ref: np.ndarray, terms, n_frames: int, dtype: str, what: str = "",
                       flags: int = 7):
    """The fused score of Eq. 7 against the oracle's.  `terms` = the oracle's raw terms (s_attn, s_temp, s_spa),
    each [B, N_v]; `flags` says which of them enter the sum.

    bf16: the stated bound, as for every other output.  fp32: Eq. 7 divides each raw term by its per-frame
    deviation, so a raw term that meets the fp32 bound (1e-5 of its own magnitude) moves its z-score by up to
    1e-5 (|x| + |mean_f|) / sigma_f, plus the z-score's own 1e-5 through sigma_f -- on an attention mass that is
    nearly uniform over a frame (|mean_f| ~ 20 sigma_f on the small configuration) that alone is 2e-4 of an O(1)
    value.  The fused element is therefore held to the error the raw terms' bound propagates to it,
    sum_terms 1e-5 ((|x| + |mean_f|) / sigma_f + |z|) + 1e-5 max(|ref|, rms(ref)); the raw terms themselves
    are held to the plain bound by the callers."""
    if dtype != "fp32":
        return assert_close(got, ref, dtype, what)
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    B, Nv = ref.shape
    bound = 1e-5 * np.maximum(np.abs(ref), float(np.sqrt(np.mean(ref ** 2))))
    for t, term in enumerate(terms):
        if not (flags >> t) & 1:
            continue
        tf = np.asarray(term, dtype=np.float64).reshape(B, n_frames, Nv // n_frames)
        mu, sg = tf.mean(-1, keepdims=True), tf.std(-1, keepdims=True)
        safe = np.where(sg > 0, sg, 1.0)
        amp = np.where(sg > 0, (np.abs(tf) + np.abs(mu)) / safe + np.abs(tf - mu) / safe, 0.0)
        bound = bound + 1e-5 * amp.reshape(B, Nv)
    err = np.abs(got - ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err / bound), err.shape)
        raise AssertionError("%s: %d of %d outside the propagated fp32 bound; worst at %s got %.9g ref %.9g (bound %.3g)"
                             % (what, int(bad.sum()), bad.size, i, got[i], ref[i], bound[i]))


def assert_indices_consistent(idx_gpu: np.ndarray, scores_ref: np.ndarray, idx_ref: np.ndarray, tol: float):
    """End-to-end selection check: GPU-scored selection may differ from the oracle-scored one only by
    tokens whose oracle score is within `tol` of the k-th largest oracle score."""
    for b in range(idx_ref.shape[0]):
        a, r = set(idx_gpu[b].tolist()), set(idx_ref[b].tolist())
        assert len(a) == idx_ref.shape[1]
        kth = np.sort(scores_ref[b])[::-1][idx_ref.shape[1] - 1]
        for j in a ^ r:
            assert abs(scores_ref[b, j] - kth) <= tol, (b, j, scores_ref[b, j], kth)
