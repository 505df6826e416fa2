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


@dataclass
class FreeRunReport:
    """Free-running comparison (no teacher forcing): every disagreement with the oracle's own sweep, by cause."""
    groups: int
    subvectors: int
    scale_mismatch: int = 0
    scale_ties: int = 0          # the oracle's fp64 sigma sits on an fp16 rounding boundary
    scale_from_inputs: int = 0   # the library's own residual has the scale the library stored
    code_mismatch: int = 0
    distance_ties: int = 0       # the library's grid point is within TIE_GAP of the oracle's, on the oracle's input
    scale_tie_codes: int = 0     # the oracle gives the library's code under the library's (tied) scale
    from_inputs: int = 0         # the gap on the oracle's input is covered by the measured difference of the inputs
    other: int = 0
    max_input_diff: float = 0.0  # largest |y_library - y_oracle| (normalised rotated units) over groups with equal scales

    def __str__(self):
        return (f"groups={self.groups} subvectors={self.subvectors} scale_mismatch={self.scale_mismatch} (boundary ties "
                f"{self.scale_ties}, from inputs {self.scale_from_inputs}) code_mismatch={self.code_mismatch} (distance ties "
                f"{self.distance_ties}, scale ties {self.scale_tie_codes}, from inputs {self.from_inputs}) other={self.other} "
                f"max input difference={self.max_input_diff:.3g}")


def classify_free_run(x, p_oracle, p_gpu, signs, codebook, gpu_codes, gpu_scales, n) -> FreeRunReport:
    """The library's codes and scales against the oracle's OWN sweep for the same raw tensor x [T, G, g].

    The two quantizers did not see the same residual: p_oracle is the prediction the oracle formed from its own
    earlier reconstructions, p_gpu the one the library formed from its own (fp32 accumulation, possibly other
    reconstructions upstream).  Every disagreement is put down to a cause, measured on the oracle's own input y_o:
      distance tie  - gap = d(y_o, C[code_gpu]) - d(y_o, C[code_oracle]) <= TIE_GAP;
      scale tie     - the group's scales are neighbours in fp16, the oracle's sigma lies within SCALE_TIE_REL of the
                      rounding boundary, and under the library's scale the oracle picks the library's code;
      from inputs   - the library minimised over y_g = y_o + dy.  d(y, C_a) - d(y, C_b) is linear in y with
                      gradient 2 (C_b - C_a), so choosing code_gpu at y_g is consistent iff
                      gap <= 2 |dy| |C[code_gpu] - C[code_oracle]| (+ TIE_GAP); dy is measured, not assumed;
      other         - none of these: a real disagreement.  Callers assert it is zero."""
    x = np.asarray(x, dtype=np.float64)
    C = np.asarray(codebook, dtype=np.float64)
    r_o, r_g = x - p_oracle, x - p_gpu
    idx_o, s16_o, d_o = O.quantize(r_o, signs, codebook)
    g_s16 = np.ascontiguousarray(gpu_scales).view(np.float16).reshape(s16_o.shape)
    g_idx = O.unpack_codes(gpu_codes, n)
    _, s16_own, d_own = O.quantize(r_g, signs, codebook)                      # the library's residual, the oracle's scale rule
    _, _, d_g = O.quantize(r_g, signs, codebook, sigma16_override=g_s16)      # ... normalised by the scale the library stored
    rep = FreeRunReport(groups=s16_o.size, subvectors=idx_o.size)
    bits16 = lambda a: a.view(np.uint16).astype(np.int64)
    sm = bits16(g_s16) != bits16(s16_o)
    rep.scale_mismatch = int(sm.sum())
    s_tie = sm & (fp16_boundary_distance(d_o.sigma) <= SCALE_TIE_REL) & (np.abs(bits16(g_s16) - bits16(s16_o)) == 1)
    own_ok = (bits16(s16_own) == bits16(g_s16)) | ((fp16_boundary_distance(d_own.sigma) <= SCALE_TIE_REL) &
                                                   (np.abs(bits16(g_s16) - bits16(s16_own)) == 1))
    s_in = sm & ~s_tie & own_ok
    rep.scale_ties, rep.scale_from_inputs = int(s_tie.sum()), int(s_in.sum())
    rep.other += int((sm & ~s_tie & ~s_in).sum())
    sub = lambda y: y.reshape(y.shape[:-1] + (y.shape[-1] // 2, 2))
    yo, yg = sub(d_o.y), sub(d_g.y)
    cm = g_idx != idx_o
    rep.code_mismatch = int(cm.sum())
    gap = ((yo - C[g_idx]) ** 2).sum(-1) - ((yo - C[idx_o]) ** 2).sum(-1)
    assert gap.min() >= -1e-12                                                 # the oracle's choice is the argmin
    d_tie = cm & (gap <= TIE_GAP)
    idx_t, _, _ = O.quantize(r_o, signs, codebook, sigma16_override=np.where(s_tie, g_s16, s16_o))
    st_codes = cm & ~d_tie & s_tie[..., None] & (idx_t == g_idx)
    dy = np.sqrt(((yg - yo) ** 2).sum(-1))
    reach = 2.0 * dy * np.sqrt(((C[g_idx] - C[idx_o]) ** 2).sum(-1)) + TIE_GAP
    f_in = cm & ~d_tie & ~st_codes & (gap <= reach)
    rep.distance_ties, rep.scale_tie_codes, rep.from_inputs = int(d_tie.sum()), int(st_codes.sum()), int(f_in.sum())
    rep.other += int((cm & ~d_tie & ~st_codes & ~f_in).sum())
    # over the groups whose scales agree (where they differ, y carries the other scale: half an fp16 ulp times |y|)
    same = ~sm
    rep.max_input_diff = float(np.abs(yg - yo)[same].max()) if same.any() else 0.0
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
