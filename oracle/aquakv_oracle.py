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
  * Sect. 3.1 footnote: Q is scale independent "due to the use of scales".

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
  * rotary embedding (Sect. 3.3 "Positional embeddings": keys are compressed
    before it): when scoring, the decoded key of token t is rotated by position
    t, coordinate d paired with d + g/2, angles from caller-supplied cos / sin
    tables; the query is taken as already rotated.

Pins (tests/test_oracle_pins.py): Hadamard orthogonality and Parseval, the
Kronecker recursion, fast-butterfly agreement, inverse round trip, exact
power-of-two scale covariance (the footnote of Sect. 3.1), zero residual round
trip, brute-force nearest codeword against the expanded inner-product form and
the Voronoi self-map, the grid's mean squared error on N(0,1) samples against
the paper's "2-bit explains about 0.89 of the variance" and the textbook
Lloyd-Max / rate-distortion bounds, bit accounting 2 + 16/1024 = 2.02 and the
predictor storage sizes of Table 1, bf16 / fp16 rounding against torch's
conversions, the predictor against identity / zero weights, closed loop
decode(encode(x)), the score identity q . iRHT(z) = RHT'(q) . z, and for the
rotary embedding: identity at position 0, norm preservation, the complex
multiplication form, and scores that depend only on the position difference.
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
    codebook: np.ndarray                 # [n, p]
    signs_k: np.ndarray                  # [kv_heads, head_dim] +-1
    signs_v: np.ndarray
    dtype: str = "bf16"                  # storage dtype of K, V, reconstructions, weights
    w_k: Optional[np.ndarray] = None     # [D, D]      None => no predictor (layer 0)
    b_k: Optional[np.ndarray] = None
    w_v: Optional[np.ndarray] = None     # [D, 2D]     inputs: [Vhat_prev, Khat]
    b_v: Optional[np.ndarray] = None
    rht_group: Optional[int] = None      # values per rotation group and scale; None => head_dim.
    #                                      The experiments of Sect. 4.1 run the backbone quantizer with
    #                                      groups of 1024 = the whole token vector across the kv heads.

    @property
    def n_codewords(self):
        return int(np.asarray(self.codebook).shape[0])

    @property
    def group(self):
        g = self.head_dim if self.rht_group is None else int(self.rht_group)
        if (self.kv_heads * self.head_dim) % g:
            raise ValueError("rht_group must divide kv_heads * head_dim")
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
    return np.asarray(signs, dtype=np.float64).reshape(layer.groups_per_token, layer.group)


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
    n = layer.n_codewords
    gshape = K.shape                                                      # [T, groups per token, group]
    shape = (T, layer.kv_heads, layer.head_dim)
    sk, sv = _group_signs(layer.signs_k, layer), _group_signs(layer.signs_v, layer)

    P_k = _key_prediction(layer, Khat_prev, T).reshape(gshape)            # K_pred
    k_idx, k_s16, k_diag = quantize(K - P_k, sk, layer.codebook)          # K_q
    Khat = round_storage(dequantize(k_idx, k_s16, sk, layer.codebook) + P_k, layer.dtype)

    P_v = _value_prediction(layer, Vhat_prev, Khat, T).reshape(gshape)    # V_pred uses Khat
    v_idx, v_s16, v_diag = quantize(V - P_v, sv, layer.codebook)          # V_q
    Vhat = round_storage(dequantize(v_idx, v_s16, sv, layer.codebook) + P_v, layer.dtype)

    return dict(k_codes=pack_codes(k_idx, n), k_scales=k_s16, v_codes=pack_codes(v_idx, n), v_scales=v_s16,
                Khat=Khat.reshape(shape), Vhat=Vhat.reshape(shape), P_k=P_k.reshape(shape), P_v=P_v.reshape(shape),
                k_idx=k_idx, v_idx=v_idx, k_diag=k_diag, v_diag=v_diag)


def decode_layer(layer: Layer, k_codes, k_scales, v_codes, v_scales, Khat_prev=None, Vhat_prev=None):
    """Alg. "decode": Khat = Q^{-1}(K_q) + f_key(Khat_prev); Vhat likewise from [Vhat_prev, Khat]."""
    k_codes = np.asarray(k_codes)
    T = k_codes.shape[0]
    n = layer.n_codewords
    shape = (T, layer.kv_heads, layer.head_dim)
    gshape = (T, layer.groups_per_token, layer.group)
    sk, sv = _group_signs(layer.signs_k, layer), _group_signs(layer.signs_v, layer)
    k_idx = unpack_codes(k_codes.reshape(T, layer.groups_per_token, -1), n)
    v_idx = unpack_codes(np.asarray(v_codes).reshape(T, layer.groups_per_token, -1), n)

    P_k = _key_prediction(layer, Khat_prev, T).reshape(gshape)
    Khat = round_storage(dequantize(k_idx, np.asarray(k_scales).reshape(T, -1), sk, layer.codebook) + P_k, layer.dtype)
    P_v = _value_prediction(layer, Vhat_prev, Khat, T).reshape(gshape)
    Vhat = round_storage(dequantize(v_idx, np.asarray(v_scales).reshape(T, -1), sv, layer.codebook) + P_v, layer.dtype)
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
    n = layer.n_codewords
    gshape = (T, layer.groups_per_token, layer.group)
    k_idx = unpack_codes(np.asarray(k_codes).reshape(T, layer.groups_per_token, -1), n)
    P_k = _key_prediction(layer, Khat_prev, T).reshape(gshape)
    Khat = round_storage(dequantize(k_idx, np.asarray(k_scales).reshape(T, -1), _group_signs(layer.signs_k, layer),
                                    layer.codebook) + P_k, layer.dtype)
    Khat = Khat.reshape(batch, seq_len, layer.kv_heads, layer.head_dim)
    if rope is not None:
        Khat = apply_rope(Khat, rope[0], rope[1])
    q_heads = q.shape[1]
    rep = q_heads // layer.kv_heads
    out = np.empty((batch, q_heads, seq_len))
    for qh in range(q_heads):
        out[:, qh, :] = np.einsum("bd,btd->bt", q[:, qh, :], Khat[:, :, qh // rep, :])
    return score_scale * out
