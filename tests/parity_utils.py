"""Shared helpers of the GPU parity tests: build the same layer for the oracle
and for the HIP library from one set of seeded arrays, and classify
disagreements on codes / scales the way the tests report them."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from oracle import aquakv_oracle as O
from paper_2501_19392_amd import synth

TIE_GAP = 1e-6          # squared-distance gap (normalised units) below which two codewords count as tied
SCALE_TIE_REL = 1e-6    # relative distance of sigma to an fp16 rounding boundary that counts as a scale tie
RTOL = {"fp32": 1e-5, "bf16": 2e-2}


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().double().cpu().numpy()


def make_layers(kv_heads, dtype, n, layer_idx=1, w_k=None, w_v=None, b_k=None, b_v=None, device="cuda", table=True,
                rht_group=None, rtn_bits=None):
    """(oracle layer, binding layer) from the same arrays.  w_* are torch fp32 [D, d_in]
    and are rounded to the storage dtype first so that both sides see identical weights.
    rtn_bits: the uniform round-to-nearest backbone instead of the grid of n points."""
    from paper_2501_19392_amd import binding as B
    g = 128
    sd = synth.torch_dtype(dtype)
    if rtn_bits is not None:
        wk = None if w_k is None else w_k.to(sd)
        wv = None if w_v is None else w_v.to(sd)
        f32 = lambda t: None if t is None else t.float()
        lo = O.Layer(kv_heads=kv_heads, head_dim=g, dtype=dtype, rtn_bits=rtn_bits, rtn_group=rht_group or 64,
                     w_k=None if wk is None else np64(wk), w_v=None if wv is None else np64(wv),
                     b_k=None if b_k is None else np64(f32(b_k)), b_v=None if b_v is None else np64(f32(b_v)))
        dev = lambda t: None if t is None else t.to(device)
        lg = B.Layer(kv_heads, g, None, None, None, sd, w_k=dev(wk), w_v=dev(wv), b_k=dev(f32(b_k)), b_v=dev(f32(b_v)),
                     rtn_bits=rtn_bits, rht_group=rht_group or 0)
        return lo, lg
    C = synth.lloyd_codebook(n)
    sk = synth.rht_signs(kv_heads, g, layer_idx, "k")
    sv = synth.rht_signs(kv_heads, g, layer_idx, "v")
    wk = None if w_k is None else w_k.to(sd)
    wv = None if w_v is None else w_v.to(sd)
    lo = O.Layer(kv_heads=kv_heads, head_dim=g, codebook=C, signs_k=sk, signs_v=sv, dtype=dtype,
                 w_k=None if wk is None else np64(wk), w_v=None if wv is None else np64(wv),
                 b_k=None if b_k is None else np64(b_k.float()), b_v=None if b_v is None else np64(b_v.float()),
                 rht_group=rht_group)
    dev = lambda t: None if t is None else t.to(device)
    Cd = torch.from_numpy(C).to(device)
    lg = B.Layer(kv_heads, g, Cd, torch.from_numpy(sk).to(device),
                 torch.from_numpy(sv).to(device), sd, w_k=dev(wk), w_v=dev(wv),
                 b_k=dev(None if b_k is None else b_k.float()), b_v=dev(None if b_v is None else b_v.float()),
                 search_table=B.build_search_table(Cd) if table else None, rht_group=rht_group or 0)
    return lo, lg


def random_weights(d_out, d_in, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(d_out, d_in, generator=g) * (scale / d_in ** 0.5)


@dataclass
class CodeReport:
    groups: int
    subvectors: int
    scale_mismatch: int = 0
    scale_ties: int = 0
    code_mismatch: int = 0
    distance_ties: int = 0
    other: int = 0

    def __str__(self):
        return (f"groups={self.groups} subvectors={self.subvectors} scale_mismatch={self.scale_mismatch} "
                f"(ties {self.scale_ties}) code_mismatch={self.code_mismatch} (distance ties {self.distance_ties}) "
                f"other={self.other}")


def fp16_boundary_distance(sigma: np.ndarray) -> np.ndarray:
    """Relative distance of each fp64 sigma to the nearest fp16 rounding boundary."""
    s16 = sigma.astype(np.float16)
    up = np.nextafter(s16, np.float16(np.inf)).astype(np.float64)
    dn = np.nextafter(s16, np.float16(-np.inf)).astype(np.float64)
    c = s16.astype(np.float64)
    d = np.minimum(np.abs(sigma - (c + up) / 2), np.abs(sigma - (c + dn) / 2))
    return d / np.maximum(sigma, 1e-300)


def compare_quantizer_outputs(residual, signs, codebook, gpu_codes, gpu_scales, n) -> CodeReport:
    """Codes and scales of the HIP path against the oracle for the same residual.

    gpu_codes: uint8 [T, H, bytes]; gpu_scales: int16/uint16 [T, H] fp16 bit patterns.
    A scale that differs must sit on an fp16 rounding boundary of the oracle's fp64 sigma
    (scale tie); its group is then re-assigned by the oracle under the GPU's scale.  A code that
    differs must be a near tie of the two best squared distances (<= TIE_GAP).  Anything else
    is `other` and the caller asserts it is zero."""
    idx_o, s16_o, diag = O.quantize(residual, signs, codebook)
    g_s16 = np.ascontiguousarray(gpu_scales).view(np.float16).reshape(s16_o.shape)
    g_idx = O.unpack_codes(gpu_codes, n)
    rep = CodeReport(groups=s16_o.size, subvectors=idx_o.size)
    sm = g_s16.view(np.uint16) != s16_o.view(np.uint16)
    rep.scale_mismatch = int(sm.sum())
    bad_scale = np.zeros_like(sm)
    if rep.scale_mismatch:
        near = fp16_boundary_distance(diag.sigma) <= SCALE_TIE_REL
        adjacent = np.abs(g_s16.view(np.uint16).astype(np.int64) - s16_o.view(np.uint16).astype(np.int64)) == 1
        ok = sm & near & adjacent
        bad_scale = sm & ~ok
        rep.scale_ties = int(ok.sum())
        rep.other += int(bad_scale.sum())
        # groups whose scale sat on a rounding boundary are re-assigned under the GPU's scale
        idx_o, _, diag = O.quantize(residual, signs, codebook, sigma16_override=np.where(ok, g_s16, s16_o))
    cm = (g_idx != idx_o) & ~bad_scale[..., None]
    rep.code_mismatch = int(cm.sum())
    ties = cm & (diag.gap <= TIE_GAP)
    rep.distance_ties = int(ties.sum())
    rep.other += int((cm & ~ties).sum())
    return rep


RTN_TIE = 1e-5         # distance of value / step (or -lo / step) to x.5 below which a rounding counts as tied


def compare_rtn_outputs(residual, gpu_codes, gpu_meta, bits, group=64) -> CodeReport:
    """Round-to-nearest backbone: codes, steps and zero points of the HIP path against the oracle, same residual.

    residual [T, D]; gpu_codes uint8 [T, ...]; gpu_meta (u)int16 [T, D/64, 2].  A step that differs must sit on an
    fp16 rounding boundary of the oracle's fp64 step, a zero point that differs on x.5; such groups are re-assigned
    by the oracle under the GPU's step / zero point.  A code that differs must be a value within RTN_TIE of a
    rounding boundary.  Anything else is `other`."""
    T = residual.shape[0]
    idx_o, s16_o, zero_o, diag = O.rtn_quantize(residual, bits, group)
    groups = s16_o.shape[-1]
    g_s16, g_zero = O.rtn_unpack_meta(np.ascontiguousarray(gpu_meta).reshape(T, groups, 2))
    g_idx = O.unpack_codes(np.ascontiguousarray(gpu_codes).reshape(T, groups, -1), 1 << bits)
    rep = CodeReport(groups=s16_o.size, subvectors=idx_o.size)
    sm = g_s16.view(np.uint16) != s16_o.view(np.uint16)
    zm = g_zero != zero_o
    rep.scale_mismatch = int((sm | zm).sum())
    bad = np.zeros_like(sm)
    if rep.scale_mismatch:
        near = fp16_boundary_distance(diag.scale) <= SCALE_TIE_REL
        adjacent = np.abs(g_s16.view(np.uint16).astype(np.int64) - s16_o.view(np.uint16).astype(np.int64)) == 1
        s_ok = sm & near & adjacent
        # the zero point is judged under the step that is finally used
        idx_o, _, zero_o, diag = O.rtn_quantize(residual, bits, group, scale16_override=np.where(s_ok, g_s16, s16_o))
        zm = g_zero != zero_o
        z_ok = zm & (diag.zero_frac <= RTN_TIE) & (np.abs(g_zero - zero_o) == 1)
        bad = (sm & ~s_ok) | (zm & ~z_ok)
        rep.scale_ties = int((s_ok | z_ok).sum())
        rep.other += int(bad.sum())
        idx_o, _, _, diag = O.rtn_quantize(residual, bits, group, scale16_override=np.where(s_ok, g_s16, s16_o),
                                           zero_override=np.where(z_ok, g_zero, zero_o))
    cm = (g_idx != idx_o) & ~bad[..., None]
    rep.code_mismatch = int(cm.sum())
    ties = cm & (diag.frac <= RTN_TIE) & (np.abs(g_idx - idx_o) == 1)
    rep.distance_ties = int(ties.sum())
    rep.other += int((cm & ~ties).sum())
    return rep


def rtn_decode(gpu_codes, gpu_meta, bits, T):
    """The oracle's inverse of stored round-to-nearest codes -> residual [T, D]."""
    meta = np.ascontiguousarray(gpu_meta).reshape(T, -1, 2)
    s16, zero = O.rtn_unpack_meta(meta)
    idx = O.unpack_codes(np.ascontiguousarray(gpu_codes).reshape(T, meta.shape[1], -1), 1 << bits)
    return O.rtn_dequantize(idx, s16, zero)


def assert_close_storage(got: torch.Tensor, want: np.ndarray, dtype: str, what: str):
    """Element-by-element: |got - want| <= rtol * (|want| + rms of want over its group of 128)."""
    g = np64(got).reshape(want.shape)
    rtol = RTOL[dtype]
    rms = np.sqrt(np.mean(want.reshape(-1, 128) ** 2, axis=1, keepdims=True)).repeat(128, axis=1).reshape(want.shape)
    bound = rtol * (np.abs(want) + rms) + 1e-30
    bad = np.abs(g - want) > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} elements outside tolerance; worst ratio " \
                          f"{float(np.max(np.abs(g - want) / bound)):.3g}"
    return float(np.max(np.abs(g - want) / bound))
