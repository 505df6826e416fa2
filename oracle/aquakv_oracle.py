"""CPU oracle for the AQUA-KV per-layer KV-cache encode / decode path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the HIP
library is checked against.  It shares no code with the HIP path, is never
imported by the product package, and may be imported only by tests, by the
smoke check and by the benchmark's cpu-baseline leg.

Everything is numpy in fp64 unless a storage precision is fixed below.  Each
function cites the passage of the AQUA-KV paper (arxiv 2501.19392) it follows:

  * Sect. 2 "Vector Quantization": the backbone quantizer Q (HIGGS): randomized
    Hadamard transform, group scales, round-to-nearest on a grid of n points in
    R^p built for normally distributed vectors (Sect. 4.1: p = 2, n = 16/64/256).
  * Sect. 3.2: linear predictors f_key (previous layer's reconstructed keys) and
    f_value (previous layer's reconstructed values, then this layer's
    reconstructed keys).
  * Appendix, Alg. "encode" and Alg. "decode": order of the steps per layer.
  * Sect. 3.1 footnote: Q does not depend on the scale of its input, because every group is normalised.
  * Sect. 4.1 "Backbone quantization": the second backbone, uniform round-to-nearest
    with per-group normalisation (groups of 64 channels of a token), rtn_quantize.

Readings taken where the paper is silent (all are also listed in the design
notes of the repository):

  * RHT: z = H_g (s * r) / sqrt(g), H_g the Sylvester Hadamard matrix in natural
    order, s a fixed +-1 vector per channel; inverse x = s * (H_g z) / sqrt(g).
    One group = one (token, kv head) vector of g = head_dim values by default;
    Layer.rht_group = kv_heads * head_dim gives the grouping of the paper's
    experiments (Sect. 4.1: groups of 1024, one 16-bit scale per group, hence
    the 2.02 bits of Table 1): the whole token vector is one group.
  * scale: sigma = sqrt(mean(z^2)) of the rotated group, stored as IEEE fp16
    (round to nearest even, clamped to the largest finite fp16); the group is
    normalised by the *stored* value; a stored zero means the group decodes to 0.
  * sub-vector i of a group is the rotated coordinates (p*i .. p*i+p-1);
    ties in the nearest-codeword search go to the lowest index.
  * codes are packed as a little-endian bit string per group, c = log2(n) bits
    per code, code i at bits [i*c, (i+1)*c).
  * predictor: y = x @ W.T + b with W stored [d_out, d_in]; fp64 accumulation,
    rounded once to fp32 (the precision the prediction is carried in);
    the reconstruction is rounded to the storage dtype (bf16 or fp32) and it is
    the rounded tensor that feeds the value predictor and the next layer.
  * layer 0 has no predictor: the prediction is zero and the tensors are
    quantized like any other residual.
  * round-to-nearest backbone: the paper names the scheme and Table 1 its size
    (2.50 bits at 2 bits and groups of 64 = 32 bits of metadata per group); taken as
    min/max over a range that always holds 0, an fp16 step and an integer zero point
    (details in rtn_quantize).
  * rotary embedding (Sect. 3.3 "Positional embeddings": keys are compressed
    before it): when scoring, the decoded key of token t is rotated by position
    t, coordinate d paired with d + g/2, angles from caller-supplied cos / sin
    tables; the query is taken as already rotated.
  * value side of attention (Alg. "Inference": the block call attends over the
    recovered keys and values; its output is the weighted sum of the values): the paper's experiments hand the decoded
    tensors to a stock attention; attn_values is that sum written out over the
    storage-rounded values of Alg. "decode", for weights the caller supplies
    (softmax_rows of the scores in the plain case), grouped-query heads mapped as
    in attn_scores.

Pins (tests/test_oracle_pins.py): Hadamard orthogonality and Parseval, the
Kronecker recursion, fast-butterfly agreement, inverse round trip, exact
power-of-two scale covariance (the footnote of Sect. 3.1), zero residual round
trip, brute-force nearest codeword against the expanded inner-product form and
the Voronoi self-map, the grid's mean squared error on N(0,1) samples against
the paper's figure for a 2-bit quantizer (about 0.89 of the variance explained) and the textbook
Lloyd-Max / rate-distortion bounds, bit accounting 2 + 16/1024 = 2.02 and the
predictor storage sizes of Table 1, bf16 / fp16 rounding against torch's
conversions, the predictor against identity / zero weights, closed loop
decode(encode(x)), the score identity q . iRHT(z) = RHT'(q) . z, and for the
rotary embedding: identity at position 0, norm preservation, the complex
multiplication form, and scores that depend only on the position difference;
for the round-to-nearest backbone: a group worked by hand, brute force over all
levels, the half-step error bound, 0 decoding to 0, group independence, the
2.50 / 2.03 bits of the paper's tables, closed loop through predictors;
for the value side: soft-max against scipy's routine, shift invariance and rows
summing to one, one-hot weights returning a decoded row, uniform weights the
mean, brute-force triple loop with the grouped-query head map, linearity in the
weights, and the full attention against torch's scaled_dot_product_attention
(also for `attention` over given keys and values, with its row statistics).
No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np

FP16_MAX = 65504.0


# --------------------------------------------------------------------------
# storage roundings
# --------------------------------------------------------------------------
def round_bf16(x):
    """Round fp64 values to the nearest bfloat16 (ties to even), returned as fp64.

    bfloat16 = 1 sign, 8 exponent, 7 mantissa bits.  Done directly from fp64 so
    that there is a single rounding.
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    a = np.abs(x)
    sub = a < 2.0 ** -126
    # subnormal range: fixed quantum 2^-133
    q = 2.0 ** -133
    out[sub] = np.rint(x[sub] / q) * q          # np.rint rounds half to even
    # normal range: keep 7 of the 52 mantissa bits
    bits = np.ascontiguousarray(x[~sub]).view(np.uint64)
    drop = np.uint64(45)
    lsb = (bits >> drop) & np.uint64(1)
    bits = bits + np.uint64((1 << 44) - 1) + lsb
    bits = bits & ~np.uint64((1 << 45) - 1)
    r = bits.view(np.float64)
    if np.any(np.abs(r) > 3.3895313892515355e38):
        raise OverflowError("value beyond the bfloat16 range")
    out[~sub] = r
    return out


def round_fp32(x):
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_storage(x, dtype: str):
    """Round to the dtype K, V and their reconstructions are stored in."""
    if dtype == "bf16":
        return round_bf16(x)
    if dtype == "fp32":
        return round_fp32(x)
    raise ValueError(dtype)


def to_fp16_scale(sigma):
    """fp64 scale -> IEEE fp16 (nearest even), clamped to the largest finite value."""
    sigma = np.minimum(np.asarray(sigma, dtype=np.float64), FP16_MAX)
    return sigma.astype(np.float16)


# --------------------------------------------------------------------------
# randomized Hadamard transform (Sect. 2, "Vector Quantization")
# --------------------------------------------------------------------------
def hadamard(g: int) -> np.ndarray:
    """Sylvester Hadamard matrix, natural order: H[i, j] = (-1)^popcount(i & j)."""
    if g < 1 or g & (g - 1):
        raise ValueError("g must be a power of two")
    i = np.arange(g, dtype=np.int64)
    a = i[:, None] & i[None, :]
    par = np.zeros_like(a)
    while np.any(a):
        par ^= a & 1
        a >>= 1
    return 1 - 2 * par


def rht(r, signs):
    """z = H_g (s * r) / sqrt(g) on the last axis (dense +-1 product, fp64)."""
    r = np.asarray(r, dtype=np.float64)
    g = r.shape[-1]
    H = hadamard(g).astype(np.float64)
    u = r * np.asarray(signs, dtype=np.float64)
    return (u @ H.T) / math.sqrt(g)


def irht(z, signs):
    """x = s * (H_g z) / sqrt(g): the inverse of rht (H is symmetric, H H = g I)."""
    z = np.asarray(z, dtype=np.float64)
    g = z.shape[-1]
    H = hadamard(g).astype(np.float64)
    return (z @ H.T) / math.sqrt(g) * np.asarray(signs, dtype=np.float64)


# --------------------------------------------------------------------------
# grid assignment, packing (Sect. 2; Sect. 4.1 for p and n)
# --------------------------------------------------------------------------
def nearest_codeword(y, codebook):
    """Index of the nearest codeword for every p-dim sub-vector.

    y: [..., m, p]; codebook: [n, p].  All n candidates are tried; the first
    (lowest) index wins a tie (np.argmin).
    Returns (idx [..., m] int64, gap [..., m]) where gap is the squared distance
    of the runner-up minus that of the winner (used only to report near ties).
    """
    y = np.asarray(y, dtype=np.float64)
    C = np.asarray(codebook, dtype=np.float64)
    d = np.zeros(y.shape[:-1] + (C.shape[0],))
    for k in range(C.shape[1]):
        d += (y[..., k, None] - C[:, k]) ** 2
    idx = np.argmin(d, axis=-1)
    if C.shape[0] > 1:
        part = np.partition(d, 1, axis=-1)
        gap = part[..., 1] - part[..., 0]
    else:
        gap = np.full(idx.shape, np.inf)
    return idx, gap


def code_bits(n_codewords: int) -> int:
    c = int(n_codewords).bit_length() - 1
    if n_codewords < 2 or (1 << c) != n_codewords:
        raise ValueError("n_codewords must be a power of two >= 2")
    return c


def pack_codes(idx, n_codewords: int) -> np.ndarray:
    """Little-endian bit string per group: code i occupies bits [i*c, (i+1)*c).

    idx: [..., m] integers < n; returns uint8 [..., m*c/8].
    """
    c = code_bits(n_codewords)
    idx = np.asarray(idx).astype(np.uint64)
    m = idx.shape[-1]
    if (m * c) % 8:
        raise ValueError("group does not fill whole bytes")
    bits = np.zeros(idx.shape[:-1] + (m * c,), dtype=np.uint8)
    for b in range(c):
        bits[..., b::c] = ((idx >> np.uint64(b)) & np.uint64(1)).astype(np.uint8)
    return np.packbits(bits, axis=-1, bitorder="little")


def unpack_codes(packed, n_codewords: int) -> np.ndarray:
    c = code_bits(n_codewords)
    bits = np.unpackbits(np.asarray(packed, dtype=np.uint8), axis=-1, bitorder="little")
    m = bits.shape[-1] // c
    idx = np.zeros(bits.shape[:-1] + (m,), dtype=np.int64)
    for b in range(c):
        idx |= bits[..., b::c].astype(np.int64) << b
    return idx


# --------------------------------------------------------------------------
# the backbone quantizer Q and its inverse
# --------------------------------------------------------------------------
@dataclass
class QuantDiag:
    """Side information for reporting ties; not part of the method."""
    sigma: np.ndarray      # fp64 scale before rounding to fp16   [T, H]
    gap: np.ndarray        # runner-up minus winner squared distance [T, H, g/p]
    y: np.ndarray          # normalised rotated values             [T, H, g]


def quantize(r, signs, codebook, sigma16_override=None):
    """Q(r): r [T, H, g] residuals, signs [H, g], codebook [n, p].

    Returns (idx [T, H, g/p] int64, sigma16 [T, H] float16, QuantDiag).
    sigma16_override (same shape as sigma16) replaces the stored scale; it
    exists so that a test can tell a scale that sat on an fp16 rounding
    boundary from any other disagreement.
    """
    r = np.asarray(r, dtype=np.float64)
    C = np.asarray(codebook, dtype=np.float64)
    p = C.shape[1]
    z = rht(r, signs)                                   # rotate
    sigma = np.sqrt(np.mean(z * z, axis=-1))            # group RMS
    sigma16 = to_fp16_scale(sigma) if sigma16_override is None else np.asarray(sigma16_override, dtype=np.float16)
    s = sigma16.astype(np.float64)[..., None]
    y = np.divide(z, s, out=np.zeros_like(z), where=s != 0)   # stored 0 => y = 0
    sub = y.reshape(y.shape[:-1] + (y.shape[-1] // p, p))
    idx, gap = nearest_codeword(sub, C)
    return idx, sigma16, QuantDiag(sigma=sigma, gap=gap, y=y)


def dequantize(idx, sigma16, signs, codebook):
    """Q^{-1}: gather codewords, rescale by the stored scale, rotate back."""
    C = np.asarray(codebook, dtype=np.float64)
    zhat = C[np.asarray(idx)]                           # [..., m, p]
    zhat = zhat.reshape(zhat.shape[:-2] + (-1,))
    zhat = zhat * np.asarray(sigma16).astype(np.float64)[..., None]
    return irht(zhat, signs)


# --------------------------------------------------------------------------
# second backbone: uniform round-to-nearest with a zero point (Sect. 4.1, "Backbone quantization")
# --------------------------------------------------------------------------
@dataclass
class RtnDiag:
    """Side information for reporting ties; not part of the method."""
    scale: np.ndarray      # fp64 step before rounding to fp16          [..., groups]
    zero_frac: np.ndarray  # distance of -lo/step to the nearest rounding boundary (x.5) [..., groups]
    frac: np.ndarray       # the same for every value / step                [..., groups, group]


def rtn_quantize(r, bits: int, group: int = 64, scale16_override=None, zero_override=None):
    """Uniform b-bit round-to-nearest with per-group min/max normalisation and an integer zero point.

    Sect. 4.1 names the scheme (simple round-to-nearest with absmax normalisation, group size 64, per-token
    compression) and Table 1 fixes its size: 2.50 bits per value at 2 bits, i.e. 32 bits of metadata per 64
    values -- a 16-bit step and a 16-bit zero point.  Reading taken: groups are `group` consecutive channels of a
    token; lo = min(0, min r), hi = max(0, max r) (the range always holds 0, which then decodes to itself);
    step = (hi - lo) / (2^b - 1) stored as fp16 (nearest even, clamped to the largest finite value); zero =
    round(-lo / step) clipped to [0, 2^b - 1]; code = clip(round(r / step) + zero, 0, 2^b - 1), rounding half to
    even, with the *stored* step.  A stored step of 0 gives codes = zero = 0.

    r: [..., d].  Returns (codes [..., d/group, group] int64, step16 [..., d/group] float16,
    zero [..., d/group] int64, RtnDiag).  scale16_override / zero_override replace the stored step / zero point;
    they exist so that a test can tell a step that sat on an fp16 rounding boundary, or a zero point that sat on
    x.5, from any other disagreement.
    """
    r = np.asarray(r, dtype=np.float64)
    L = (1 << bits) - 1
    x = r.reshape(r.shape[:-1] + (r.shape[-1] // group, group))
    lo = np.minimum(x.min(axis=-1), 0.0)
    hi = np.maximum(x.max(axis=-1), 0.0)
    step = (hi - lo) / L
    step16 = to_fp16_scale(step) if scale16_override is None else np.asarray(scale16_override, dtype=np.float16)
    s = step16.astype(np.float64)
    ok = s > 0
    zf = np.divide(-lo, s, out=np.zeros_like(s), where=ok)
    zero = np.clip(np.rint(zf), 0, L).astype(np.int64) if zero_override is None else np.asarray(zero_override, dtype=np.int64)
    y = np.divide(x, s[..., None], out=np.zeros_like(x), where=ok[..., None])
    codes = np.clip(np.rint(y).astype(np.int64) + zero[..., None], 0, L)
    half = lambda a: np.abs(np.abs(a - np.floor(a)) - 0.5)
    return codes, step16, zero, RtnDiag(scale=step, zero_frac=half(zf), frac=half(y))


def rtn_dequantize(codes, step16, zero):
    """(code - zero) * step, [..., groups, group] -> [..., groups * group]."""
    codes = np.asarray(codes, dtype=np.float64)
    out = (codes - np.asarray(zero, dtype=np.float64)[..., None]) * np.asarray(step16).astype(np.float64)[..., None]
    return out.reshape(out.shape[:-2] + (-1,))


def rtn_pack_meta(step16, zero) -> np.ndarray:
    """Per group (fp16 bits of the step, zero point) as uint16 [..., groups, 2]."""
    return np.stack([np.asarray(step16, dtype=np.float16).view(np.uint16), np.asarray(zero).astype(np.uint16)], axis=-1)


def rtn_unpack_meta(meta):
    meta = np.ascontiguousarray(meta).view(np.uint16)
    return np.ascontiguousarray(meta[..., 0]).view(np.float16), meta[..., 1].astype(np.int64)


# --------------------------------------------------------------------------
# predictors (Sect. 3.2) and the per-layer procedures (Alg. "encode"/"decode")
# --------------------------------------------------------------------------
def predict(x, W, b=None):
    """f(x) = x W^T + b.  W is [d_out, d_in]; fp64 accumulate, rounded to fp32."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)
    return round_fp32(y)


@dataclass
class Layer:
    """One layer's fixed parameters (the REQUIRE lines of Alg. encode/decode)."""
    kv_heads: int
    head_dim: int
    codebook: Optional[np.ndarray] = None    # [n, p]                        (grid backbone)
    signs_k: Optional[np.ndarray] = None     # [kv_heads, head_dim] +-1      (grid backbone)
    signs_v: Optional[np.ndarray] = None
    dtype: str = "bf16"                  # storage dtype of K, V, reconstructions, weights
    w_k: Optional[np.ndarray] = None     # [D, D]      None => no predictor (layer 0)
    b_k: Optional[np.ndarray] = None
    w_v: Optional[np.ndarray] = None     # [D, 2D]     inputs: [Vhat_prev, Khat]
    b_v: Optional[np.ndarray] = None
    rht_group: Optional[int] = None      # values per rotation group and scale; None => head_dim.
    #                                      The experiments of Sect. 4.1 run the backbone quantizer with
    #                                      groups of 1024 = the whole token vector across the kv heads.
    rtn_bits: Optional[int] = None       # set => the uniform round-to-nearest backbone (rtn_quantize) with this many
    rtn_group: int = 64                  #        bits and groups of rtn_group consecutive channels; no grid, no signs

    @property
    def n_codewords(self):
        if self.rtn_bits is not None:
            return 1 << self.rtn_bits
        return int(np.asarray(self.codebook).shape[0])

    @property
    def group(self):
        if self.rtn_bits is not None:
            g = int(self.rtn_group)
        else:
            g = self.head_dim if self.rht_group is None else int(self.rht_group)
        if (self.kv_heads * self.head_dim) % g:
            raise ValueError("the group size must divide kv_heads * head_dim")
        return g

    @property
    def groups_per_token(self):
        return self.kv_heads * self.head_dim // self.group


def _as_groups(x, layer: Layer):
    """[T, ...] -> [T, groups per token, group]: the token vector (kv heads side by side) cut into rotation groups."""
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    return x.reshape(T, layer.groups_per_token, layer.group)


def _group_signs(signs, layer: Layer):
    if layer.rtn_bits is not None:
        return None
    return np.asarray(signs, dtype=np.float64).reshape(layer.groups_per_token, layer.group)


def _quantize_residual(layer: Layer, r, signs):
    """The layer's backbone Q and its inverse on residual groups r [T, groups per token, group].
    Returns (packed codes, stored scales, code indices, diag, Q^-1(Q(r)) shaped like r)."""
    n = layer.n_codewords
    if layer.rtn_bits is not None:
        T = r.shape[0]
        idx, step16, zero, diag = rtn_quantize(r.reshape(T, -1), layer.rtn_bits, layer.group)
        return pack_codes(idx, n), rtn_pack_meta(step16, zero), idx, diag, rtn_dequantize(idx, step16, zero).reshape(r.shape)
    idx, s16, diag = quantize(r, signs, layer.codebook)
    return pack_codes(idx, n), s16, idx, diag, dequantize(idx, s16, signs, layer.codebook)


def _dequantize_stored(layer: Layer, codes, scales, signs, T):
    """Q^-1 of stored codes and scales -> residual groups [T, groups per token, group]."""
    idx = unpack_codes(np.asarray(codes).reshape(T, layer.groups_per_token, -1), layer.n_codewords)
    if layer.rtn_bits is not None:
        step16, zero = rtn_unpack_meta(np.asarray(scales).reshape(T, layer.groups_per_token, 2))
        return rtn_dequantize(idx, step16, zero).reshape(T, layer.groups_per_token, layer.group)
    return dequantize(idx, np.asarray(scales).reshape(T, -1), signs, layer.codebook)


def _key_prediction(layer: Layer, Khat_prev, T):
    D = layer.kv_heads * layer.head_dim
    if layer.w_k is None:
        return np.zeros((T, D))
    return predict(np.asarray(Khat_prev, dtype=np.float64).reshape(T, -1), layer.w_k, layer.b_k)


def _value_prediction(layer: Layer, Vhat_prev, Khat, T):
    D = layer.kv_heads * layer.head_dim
    if layer.w_v is None:
        return np.zeros((T, D))
    # concatenation order: previous values first, then the current keys
    x = np.concatenate([np.asarray(Vhat_prev, dtype=np.float64).reshape(T, -1),
                        np.asarray(Khat, dtype=np.float64).reshape(T, -1)], axis=1)
    return predict(x, layer.w_v, layer.b_v)


def encode_layer(layer: Layer, K, V, Khat_prev=None, Vhat_prev=None):
    """Alg. "encode", with the reconstructions the inference loop needs next.

    K, V: [T, H, g] holding storage-dtype values.  Returns a dict with
    k_codes/v_codes (uint8 [T, groups per token, group*c/(8p)]), k_scales/v_scales (float16
    [T, groups per token]; groups per token = H unless the layer sets rht_group),
    Khat/Vhat (fp64 arrays holding storage-dtype values), P_k/P_v, and the
    QuantDiag of both tensors.
    """
    K = _as_groups(K, layer)
    V = _as_groups(V, layer)
    T = K.shape[0]
    gshape = K.shape                                                      # [T, groups per token, group]
    shape = (T, layer.kv_heads, layer.head_dim)
    sk, sv = _group_signs(layer.signs_k, layer), _group_signs(layer.signs_v, layer)

    P_k = _key_prediction(layer, Khat_prev, T).reshape(gshape)            # K_pred
    k_codes, k_scales, k_idx, k_diag, k_rhat = _quantize_residual(layer, K - P_k, sk)     # K_q
    Khat = round_storage(k_rhat + P_k, layer.dtype)

    P_v = _value_prediction(layer, Vhat_prev, Khat, T).reshape(gshape)    # V_pred uses Khat
    v_codes, v_scales, v_idx, v_diag, v_rhat = _quantize_residual(layer, V - P_v, sv)     # V_q
    Vhat = round_storage(v_rhat + P_v, layer.dtype)

    return dict(k_codes=k_codes, k_scales=k_scales, v_codes=v_codes, v_scales=v_scales,
                Khat=Khat.reshape(shape), Vhat=Vhat.reshape(shape), P_k=P_k.reshape(shape), P_v=P_v.reshape(shape),
                k_idx=k_idx, v_idx=v_idx, k_diag=k_diag, v_diag=v_diag)


def decode_layer(layer: Layer, k_codes, k_scales, v_codes, v_scales, Khat_prev=None, Vhat_prev=None):
    """Alg. "decode": Khat = Q^{-1}(K_q) + f_key(Khat_prev); Vhat likewise from [Vhat_prev, Khat]."""
    k_codes = np.asarray(k_codes)
    T = k_codes.shape[0]
    shape = (T, layer.kv_heads, layer.head_dim)
    gshape = (T, layer.groups_per_token, layer.group)
    sk, sv = _group_signs(layer.signs_k, layer), _group_signs(layer.signs_v, layer)

    P_k = _key_prediction(layer, Khat_prev, T).reshape(gshape)
    Khat = round_storage(_dequantize_stored(layer, k_codes, k_scales, sk, T) + P_k, layer.dtype)
    P_v = _value_prediction(layer, Vhat_prev, Khat, T).reshape(gshape)
    Vhat = round_storage(_dequantize_stored(layer, v_codes, v_scales, sv, T) + P_v, layer.dtype)
    return Khat.reshape(shape), Vhat.reshape(shape)


def rope_tables(seq_len: int, head_dim: int, base: float = 10000.0):
    """cos / sin of the rotary angles, [seq_len, head_dim/2]: angle(t, i) = t * base^(-2i/head_dim)
    (RoFormer; what the models of Sect. 4 of the paper use), rounded to fp32 like the tables a caller passes."""
    half = head_dim // 2
    inv_freq = base ** (-np.arange(half, dtype=np.float64) * 2.0 / head_dim)
    ang = np.arange(seq_len, dtype=np.float64)[:, None] * inv_freq[None, :]
    return round_fp32(np.cos(ang)), round_fp32(np.sin(ang))


def apply_rope(x, cos, sin):
    """Rotary embedding of x[..., t, :, g] by per-token tables cos, sin [t, g/2]: coordinate pairs (d, d + g/2)
    are rotated by the token's angle (the "rotate half" pairing of the model implementation the paper runs on,
    Sect. 4.3): x'_d = x_d cos - x_{d+g/2} sin, x'_{d+g/2} = x_{d+g/2} cos + x_d sin."""
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    c = np.asarray(cos, dtype=np.float64)[:, None, :]
    s_ = np.asarray(sin, dtype=np.float64)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s_, hi * c + lo * s_], axis=-1)


def attn_scores(layer: Layer, batch: int, seq_len: int, q, k_codes, k_scales, Khat_prev=None, score_scale=1.0, rope=None):
    """scores[b, qh, t] = score_scale * q[b, qh, :] . Khat[b, t, kvh(qh), :].

    Khat is the storage-rounded reconstruction of Alg. "decode" for the keys;
    query head qh reads kv head qh // (q_heads // kv_heads).
    q: [batch, q_heads, g]; codes/scales/Khat_prev are [batch*seq_len, H, ...].
    rope = (cos, sin), each [seq_len, g/2]: the cache holds keys from before the rotary embedding
    (Sect. 3.3 "Positional embeddings"), so the key of token t is rotated by position t after decoding
    and before the dot product; q is taken as already rotated.  None: no rotary embedding.
    """
    q = np.asarray(q, dtype=np.float64)
    T = batch * seq_len
    gshape = (T, layer.groups_per_token, layer.group)
    P_k = _key_prediction(layer, Khat_prev, T).reshape(gshape)
    Khat = round_storage(_dequantize_stored(layer, k_codes, k_scales, _group_signs(layer.signs_k, layer), T) + P_k,
                         layer.dtype)
    Khat = Khat.reshape(batch, seq_len, layer.kv_heads, layer.head_dim)
    if rope is not None:
        Khat = apply_rope(Khat, rope[0], rope[1])
    q_heads = q.shape[1]
    rep = q_heads // layer.kv_heads
    out = np.empty((batch, q_heads, seq_len))
    for qh in range(q_heads):
        out[:, qh, :] = np.einsum("bd,btd->bt", q[:, qh, :], Khat[:, :, qh // rep, :])
    return score_scale * out


def softmax_rows(scores):
    """Soft-max over the last axis: p = exp(s - max s) / sum exp(s - max s) (the attention weights of the
    block call in Alg. "Inference"; subtracting the row maximum changes nothing mathematically)."""
    s = np.asarray(scores, dtype=np.float64)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attn_values(layer: Layer, batch: int, seq_len: int, weights, v_codes, v_scales, Vhat_prev=None, Khat=None):
    """out[b, qh, :] = sum_t weights[b, qh, t] * Vhat[b, t, kvh(qh), :]  and Vhat itself.

    Vhat is the storage-rounded reconstruction of the values of Alg. "decode" (second line:
    Q^{-1}(V_q) + f_value([Vhat_prev; Khat])); query head qh reads kv head qh // (q_heads // kv_heads).
    The weighted sum is the value side of attention (block call of Alg. "Inference"): with weights = softmax_rows(scores) it is
    the attention output over the cached tokens.  weights: [batch, q_heads, seq_len], any real numbers.
    Returns (out [batch, q_heads, head_dim], Vhat [batch*seq_len, kv_heads, head_dim]).
    """
    w = np.asarray(weights, dtype=np.float64)
    T = batch * seq_len
    gshape = (T, layer.groups_per_token, layer.group)
    P_v = _value_prediction(layer, Vhat_prev, Khat, T).reshape(gshape)
    Vhat = round_storage(_dequantize_stored(layer, v_codes, v_scales, _group_signs(layer.signs_v, layer), T) + P_v,
                         layer.dtype)
    Vhat = Vhat.reshape(batch, seq_len, layer.kv_heads, layer.head_dim)
    q_heads = w.shape[1]
    rep = q_heads // layer.kv_heads
    out = np.empty((batch, q_heads, layer.head_dim))
    for qh in range(q_heads):
        out[:, qh, :] = np.einsum("bt,btd->bd", w[:, qh, :], Vhat[:, :, qh // rep, :])
    return out, Vhat.reshape(T, layer.kv_heads, layer.head_dim)


def attention(q, K, V, score_scale=1.0, rope=None):
    """Attention of one query per sequence and query head over given keys and values (the block call of
    Alg. "Inference" for one new token): scores s[b, qh, t] = score_scale * q[b, qh] . K[b, t, kvh(qh)],
    out[b, qh] = sum_t softmax_t(s)[t] * V[b, t, kvh(qh)], query head qh reading kv head qh // (q_heads // kv_heads).
    q: [batch, q_heads, g]; K, V: [batch, tokens, kv_heads, g].
    rope = (cos, sin), each [tokens, g/2]: the keys are held from before the rotary embedding (Sect. 3.3) and key t is
    rotated by row t of the tables first (apply_rope); q is taken as already rotated.
    Returns (out, M, L) with M the row maximum of s and L = sum_t exp(s - M).
    """
    q, K, V = (np.asarray(a, dtype=np.float64) for a in (q, K, V))
    if rope is not None:
        K = apply_rope(K, rope[0], rope[1])
    batch, q_heads, _ = q.shape
    rep = q_heads // K.shape[2]
    out = np.empty_like(q)
    M = np.empty((batch, q_heads))
    L = np.empty((batch, q_heads))
    for qh in range(q_heads):
        s = score_scale * np.einsum("bd,btd->bt", q[:, qh], K[:, :, qh // rep])
        M[:, qh] = s.max(axis=1)
        e = np.exp(s - M[:, qh, None])
        L[:, qh] = e.sum(axis=1)
        out[:, qh] = np.einsum("bt,btd->bd", e / L[:, qh, None], V[:, :, qh // rep])
    return out, M, L
