"""ctypes binding of libaquakv.so: same names as the C ABI (include/aquakv.h),
argument marshalling only.  Tensors are torch tensors on the GPU (torch is used
for device memory and streams); every step of the path runs in the HIP kernels.

Importing this module without the built library raises: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaquakv.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2501_19392_amd.build` "
        "(or __graft_entry__.build()); there is no CPU fallback")

_lib = ctypes.CDLL(LIB_PATH)

AQUAKV_OK, AQUAKV_EINVAL, AQUAKV_ENULL, AQUAKV_EALIGN, AQUAKV_EUNSUPPORTED, AQUAKV_EWORKSPACE, AQUAKV_EHIP = (
    0, -1, -2, -3, -4, -5, -6)
AQUAKV_BF16, AQUAKV_FP32 = 0, 1
AQUAKV_KEY, AQUAKV_VALUE = 0, 1

# rotation groups of 1024: predictor and quantizer of the encoder run as one kernel (bench.py labels its entries by it)
WIDE_ENCODE_FUSED = True

EXPORTS = [
    "aquakv_version", "aquakv_status_string", "aquakv_last_error", "aquakv_workspace_bytes", "aquakv_fused_tile_heads",
    "aquakv_search_table_bytes", "aquakv_build_search_table",
    "aquakv_predict", "aquakv_quantize", "aquakv_dequantize",
    "aquakv_encode_layer", "aquakv_decode_layer", "aquakv_decode_attn_scores",
    "aquakv_scores_workspace_bytes", "aquakv_decode_attn_scores_rope",
    "aquakv_decode_attn_scores_folded", "aquakv_decode_attn_scores_folded_static",
    "aquakv_encode_keys", "aquakv_encode_values", "aquakv_decode_values",
    "aquakv_fit_workspace_bytes", "aquakv_fit_predictor",
    "aquakv_softmax", "aquakv_weighted_workspace_bytes", "aquakv_decode_values_weighted", "aquakv_decode_values_attend",
    "aquakv_attend_raw",
]


class aquakv_layer(ctypes.Structure):
    _fields_ = [
        ("kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("vq_dim", ctypes.c_int32),
        ("n_codewords", ctypes.c_int32), ("dtype", ctypes.c_int32), ("d_in_k", ctypes.c_int32),
        ("d_in_v", ctypes.c_int32), ("rht_group", ctypes.c_int32),
        ("codebook", ctypes.c_void_p), ("signs_k", ctypes.c_void_p), ("signs_v", ctypes.c_void_p),
        ("w_k", ctypes.c_void_p), ("b_k", ctypes.c_void_p), ("w_v", ctypes.c_void_p), ("b_v", ctypes.c_void_p),
        ("search_table", ctypes.c_void_p),
    ]


_P = ctypes.c_void_p
_LP = ctypes.POINTER(aquakv_layer)
_lib.aquakv_version.restype = ctypes.c_int
_lib.aquakv_status_string.restype = ctypes.c_char_p
_lib.aquakv_status_string.argtypes = [ctypes.c_int]
_lib.aquakv_last_error.restype = ctypes.c_char_p
_lib.aquakv_workspace_bytes.restype = ctypes.c_size_t
_lib.aquakv_workspace_bytes.argtypes = [_LP, ctypes.c_int64]
_lib.aquakv_fused_tile_heads.restype = ctypes.c_int
_lib.aquakv_fused_tile_heads.argtypes = [_LP, ctypes.c_int64]
_lib.aquakv_scores_workspace_bytes.restype = ctypes.c_size_t
_lib.aquakv_scores_workspace_bytes.argtypes = [_LP, ctypes.c_int32, ctypes.c_int32]
_lib.aquakv_search_table_bytes.restype = ctypes.c_size_t
_lib.aquakv_search_table_bytes.argtypes = [ctypes.c_int32]
_lib.aquakv_build_search_table.restype = ctypes.c_int
_lib.aquakv_build_search_table.argtypes = [_P, ctypes.c_int32, ctypes.c_int32, _P, _P]
_lib.aquakv_predict.argtypes = [_LP, ctypes.c_int, ctypes.c_int64, _P, _P, _P, _P]
_lib.aquakv_quantize.argtypes = [_LP, ctypes.c_int, ctypes.c_int64, _P, _P, _P, _P, _P, _P]
_lib.aquakv_dequantize.argtypes = [_LP, ctypes.c_int, ctypes.c_int64, _P, _P, _P, _P, _P]
_lib.aquakv_encode_layer.argtypes = [_LP, ctypes.c_int64] + [_P] * 11 + [ctypes.c_size_t, _P]
_lib.aquakv_decode_layer.argtypes = [_LP, ctypes.c_int64] + [_P] * 9 + [ctypes.c_size_t, _P]
_lib.aquakv_decode_attn_scores.argtypes = ([_LP, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _P, _P, _P, _P,
                                            ctypes.c_float, _P, _P, _P, ctypes.c_size_t, _P])
_lib.aquakv_decode_attn_scores_rope.argtypes = ([_LP, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _P, _P, _P, _P, _P, _P,
                                                 ctypes.c_float, _P, _P, _P, ctypes.c_size_t, _P])
_lib.aquakv_decode_attn_scores_folded.argtypes = ([_LP, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _P, _P, _P, _P,
                                                   ctypes.c_float, _P, _P, ctypes.c_size_t, _P])
_lib.aquakv_decode_attn_scores_folded_static.argtypes = ([_LP, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _P, _P, _P, _P,
                                                          ctypes.c_float, _P, _P])
_lib.aquakv_encode_keys.argtypes = [_LP, ctypes.c_int64] + [_P] * 6 + [ctypes.c_size_t, _P]
_lib.aquakv_encode_values.argtypes = [_LP, ctypes.c_int64] + [_P] * 7 + [ctypes.c_size_t, _P]
_lib.aquakv_decode_values.argtypes = [_LP, ctypes.c_int64] + [_P] * 6 + [ctypes.c_size_t, _P]
_lib.aquakv_fit_workspace_bytes.restype = ctypes.c_size_t
_lib.aquakv_fit_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
_lib.aquakv_fit_predictor.argtypes = [ctypes.c_int32, ctypes.c_int64, _P, ctypes.c_int32, _P, ctypes.c_int32, _P, ctypes.c_int32,
                                      ctypes.c_double, _P, _P, _P, _P, ctypes.c_size_t, _P]
_lib.aquakv_softmax.argtypes = [ctypes.c_int64, ctypes.c_int64, _P, _P, _P]
_lib.aquakv_weighted_workspace_bytes.restype = ctypes.c_size_t
_lib.aquakv_weighted_workspace_bytes.argtypes = [_LP, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
_lib.aquakv_decode_values_weighted.argtypes = [_LP, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32] + [_P] * 8 + [ctypes.c_size_t, _P]
_lib.aquakv_decode_values_attend.argtypes = [_LP, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32] + [_P] * 9 + [ctypes.c_size_t, _P]
_lib.aquakv_attend_raw.argtypes = [ctypes.c_int32] * 5 + [_P, _P, _P, _P, _P, ctypes.c_float, _P, _P, ctypes.c_int32, _P]
for _n in ("aquakv_attend_raw", "aquakv_softmax", "aquakv_decode_values_weighted", "aquakv_decode_values_attend", "aquakv_predict", "aquakv_quantize", "aquakv_dequantize", "aquakv_encode_layer", "aquakv_decode_layer",
           "aquakv_decode_attn_scores", "aquakv_decode_attn_scores_rope", "aquakv_decode_attn_scores_folded",
           "aquakv_decode_attn_scores_folded_static", "aquakv_encode_keys", "aquakv_encode_values",
           "aquakv_decode_values", "aquakv_fit_predictor"):
    getattr(_lib, _n).restype = ctypes.c_int


class AquaKVError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"{aquakv_status_string(status)} ({status}): {aquakv_last_error()}")


def _check(status: int) -> None:
    if status != AQUAKV_OK:
        raise AquaKVError(status)


def _ptr(x):
    """None -> NULL, int -> that address, tensor -> its data pointer (must be contiguous)."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    if not x.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(x.data_ptr())


def _stream(stream):
    if stream is None:
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream) if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.bfloat16:
        return AQUAKV_BF16
    if t == torch.float32:
        return AQUAKV_FP32
    raise ValueError(f"unsupported storage dtype {t}")


class Layer:
    """Owns the device tensors of one layer's parameters and the C struct that points at them."""

    def __init__(self, kv_heads: int, head_dim: int, codebook: Optional[torch.Tensor], signs_k: Optional[torch.Tensor],
                 signs_v: Optional[torch.Tensor], dtype: torch.dtype, w_k: Optional[torch.Tensor] = None,
                 w_v: Optional[torch.Tensor] = None, b_k: Optional[torch.Tensor] = None,
                 b_v: Optional[torch.Tensor] = None, search_table: Optional[torch.Tensor] = None, rht_group: int = 0,
                 rtn_bits: Optional[int] = None):
        """rtn_bits = 2 or 4 selects the uniform round-to-nearest backbone (vq_dim = 1, groups of 64): codebook,
        signs and search_table are then None."""
        self.kv_heads, self.head_dim, self.dtype = kv_heads, head_dim, dtype
        self.rtn_bits = rtn_bits
        self.d = kv_heads * head_dim
        if rtn_bits is not None:
            self.rht_group = rht_group or 64            # values per group of the round-to-nearest backbone
            self.codebook = self.signs_k = self.signs_v = None
            self.n_codewords, self.vq_dim = 1 << rtn_bits, 1
        else:
            self.rht_group = rht_group or head_dim      # values per rotation group and scale
            self.codebook = codebook.to(torch.float32).contiguous()
            self.signs_k = signs_k.to(torch.int8).contiguous().reshape(-1)
            self.signs_v = signs_v.to(torch.int8).contiguous().reshape(-1)
            self.n_codewords, self.vq_dim = self.codebook.shape
        self.w_k = None if w_k is None else w_k.to(dtype).contiguous()
        self.w_v = None if w_v is None else w_v.to(dtype).contiguous()
        self.b_k = None if b_k is None else b_k.to(torch.float32).contiguous()
        self.b_v = None if b_v is None else b_v.to(torch.float32).contiguous()
        self.search_table = search_table
        if self.w_k is not None and self.w_k.shape[0] != self.d:
            raise ValueError("w_k must be [D, d_in_k]")
        if self.w_v is not None and self.w_v.shape[0] != self.d:
            raise ValueError("w_v must be [D, d_in_v]")
        self.c = aquakv_layer(
            kv_heads=kv_heads, head_dim=head_dim, vq_dim=self.vq_dim, n_codewords=self.n_codewords,
            dtype=_dtype_code(dtype), d_in_k=0 if self.w_k is None else self.w_k.shape[1],
            d_in_v=0 if self.w_v is None else self.w_v.shape[1], rht_group=rht_group,
            codebook=None if self.codebook is None else self.codebook.data_ptr(),
            signs_k=None if self.signs_k is None else self.signs_k.data_ptr(),
            signs_v=None if self.signs_v is None else self.signs_v.data_ptr(),
            w_k=None if self.w_k is None else self.w_k.data_ptr(),
            b_k=None if self.b_k is None else self.b_k.data_ptr(),
            w_v=None if self.w_v is None else self.w_v.data_ptr(),
            b_v=None if self.b_v is None else self.b_v.data_ptr(),
            search_table=None if search_table is None else search_table.data_ptr())

    @property
    def code_bits(self) -> int:
        return int(self.n_codewords).bit_length() - 1

    @property
    def code_bytes_per_group(self) -> int:
        return self.head_dim // self.vq_dim * self.code_bits // 8

    @property
    def scale_words_per_group(self) -> int:
        """uint16 words stored per group: the fp16 scale; for the round-to-nearest backbone (fp16 step, zero point)."""
        return 1 if self.rtn_bits is None else 2

    def alloc_codes(self, tokens: int, device="cuda"):
        codes = torch.empty(tokens, self.kv_heads, self.code_bytes_per_group, dtype=torch.uint8, device=device)
        groups = self.d // self.rht_group
        shape = (tokens, groups) if self.rtn_bits is None else (tokens, groups, 2)
        scales = torch.empty(*shape, dtype=torch.int16, device=device)   # fp16 bit patterns (and zero points)
        return codes, scales

    def alloc_kv(self, tokens: int, device="cuda"):
        return torch.empty(tokens, self.kv_heads, self.head_dim, dtype=self.dtype, device=device)

    def alloc_workspace(self, tokens: int, device="cuda"):
        return torch.empty(max(aquakv_workspace_bytes(self, tokens), 16), dtype=torch.uint8, device=device)

    def alloc_scores_workspace(self, batch: int, q_heads: int, device="cuda"):
        """Workspace of aquakv_decode_attn_scores_folded (16 bytes if the layer has no folded form)."""
        return torch.empty(max(aquakv_scores_workspace_bytes(self, batch, q_heads), 16), dtype=torch.uint8, device=device)

    def alloc_weighted_workspace(self, batch: int, seq_len: int, q_heads: int, device="cuda"):
        """Workspace of aquakv_decode_values_weighted / aquakv_decode_values_attend."""
        return torch.empty(max(aquakv_weighted_workspace_bytes(self, batch, seq_len, q_heads), 16), dtype=torch.uint8,
                           device=device)


def _layer_ref(layer):
    return ctypes.byref(layer.c if isinstance(layer, Layer) else layer)


# ---------------------------------------------------------------- the C ABI, same names
def aquakv_version() -> int:
    return _lib.aquakv_version()


def aquakv_status_string(status: int) -> str:
    return _lib.aquakv_status_string(status).decode()


def aquakv_last_error() -> str:
    return _lib.aquakv_last_error().decode()


def aquakv_workspace_bytes(layer, tokens: int) -> int:
    return int(_lib.aquakv_workspace_bytes(_layer_ref(layer), tokens))


def aquakv_fused_tile_heads(layer, tokens: int) -> int:
    return int(_lib.aquakv_fused_tile_heads(_layer_ref(layer), tokens))


def aquakv_scores_workspace_bytes(layer, batch: int, q_heads: int) -> int:
    return int(_lib.aquakv_scores_workspace_bytes(_layer_ref(layer), batch, q_heads))


def aquakv_search_table_bytes(n_codewords: int) -> int:
    return int(_lib.aquakv_search_table_bytes(n_codewords))


def aquakv_build_search_table(codebook, vq_dim: int, n_codewords: int, table, stream=None) -> None:
    _check(_lib.aquakv_build_search_table(_ptr(codebook), vq_dim, n_codewords, _ptr(table), _stream(stream)))


def build_search_table(codebook: torch.Tensor) -> torch.Tensor:
    """Allocates and fills the search table for a [n, 2] fp32 device codebook."""
    n, p = codebook.shape
    table = torch.empty(aquakv_search_table_bytes(n), dtype=torch.uint8, device=codebook.device)
    aquakv_build_search_table(codebook.to(torch.float32).contiguous(), p, n, table)
    return table


def aquakv_predict(layer, which: int, tokens: int, x0, x1, P, stream=None) -> None:
    _check(_lib.aquakv_predict(_layer_ref(layer), which, tokens, _ptr(x0), _ptr(x1), _ptr(P), _stream(stream)))


def aquakv_quantize(layer, which: int, tokens: int, X, P, codes, scales, Xhat, stream=None) -> None:
    _check(_lib.aquakv_quantize(_layer_ref(layer), which, tokens, _ptr(X), _ptr(P), _ptr(codes), _ptr(scales),
                                _ptr(Xhat), _stream(stream)))


def aquakv_dequantize(layer, which: int, tokens: int, codes, scales, P, Xhat, stream=None) -> None:
    _check(_lib.aquakv_dequantize(_layer_ref(layer), which, tokens, _ptr(codes), _ptr(scales), _ptr(P), _ptr(Xhat),
                                  _stream(stream)))


def _ws(workspace):
    if workspace is None:
        return None, 0
    if isinstance(workspace, tuple):
        return ctypes.c_void_p(workspace[0]), workspace[1]
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def aquakv_encode_layer(layer, tokens: int, K, V, Khat_prev, Vhat_prev, k_codes, k_scales, v_codes, v_scales,
                        Khat, Vhat, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_encode_layer(_layer_ref(layer), tokens, _ptr(K), _ptr(V), _ptr(Khat_prev), _ptr(Vhat_prev),
                                    _ptr(k_codes), _ptr(k_scales), _ptr(v_codes), _ptr(v_scales), _ptr(Khat),
                                    _ptr(Vhat), ws, nbytes, _stream(stream)))


def aquakv_decode_layer(layer, tokens: int, k_codes, k_scales, v_codes, v_scales, Khat_prev, Vhat_prev, Khat, Vhat,
                        workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_decode_layer(_layer_ref(layer), tokens, _ptr(k_codes), _ptr(k_scales), _ptr(v_codes),
                                    _ptr(v_scales), _ptr(Khat_prev), _ptr(Vhat_prev), _ptr(Khat), _ptr(Vhat),
                                    ws, nbytes, _stream(stream)))


def aquakv_encode_keys(layer, tokens: int, K, Khat_prev, k_codes, k_scales, Khat, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_encode_keys(_layer_ref(layer), tokens, _ptr(K), _ptr(Khat_prev), _ptr(k_codes), _ptr(k_scales),
                                   _ptr(Khat), ws, nbytes, _stream(stream)))


def aquakv_encode_values(layer, tokens: int, V, Vhat_prev, Khat, v_codes, v_scales, Vhat, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_encode_values(_layer_ref(layer), tokens, _ptr(V), _ptr(Vhat_prev), _ptr(Khat), _ptr(v_codes),
                                     _ptr(v_scales), _ptr(Vhat), ws, nbytes, _stream(stream)))


def aquakv_decode_values(layer, tokens: int, v_codes, v_scales, Vhat_prev, Khat, Vhat, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_decode_values(_layer_ref(layer), tokens, _ptr(v_codes), _ptr(v_scales), _ptr(Vhat_prev), _ptr(Khat),
                                     _ptr(Vhat), ws, nbytes, _stream(stream)))


def aquakv_softmax(rows: int, n: int, scores, probs, stream=None) -> None:
    _check(_lib.aquakv_softmax(rows, n, _ptr(scores), _ptr(probs), _stream(stream)))


def aquakv_weighted_workspace_bytes(layer, batch: int, seq_len: int, q_heads: int) -> int:
    return _lib.aquakv_weighted_workspace_bytes(_layer_ref(layer), batch, seq_len, q_heads)


def aquakv_decode_values_weighted(layer, batch: int, seq_len: int, q_heads: int, v_codes, v_scales, Vhat_prev, Khat,
                                  weights, Vhat, out, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_decode_values_weighted(_layer_ref(layer), batch, seq_len, q_heads, _ptr(v_codes), _ptr(v_scales),
                                              _ptr(Vhat_prev), _ptr(Khat), _ptr(weights), _ptr(Vhat), _ptr(out), ws,
                                              nbytes, _stream(stream)))


def aquakv_decode_values_attend(layer, batch: int, seq_len: int, q_heads: int, v_codes, v_scales, Vhat_prev, Khat,
                                scores, Vhat, out, row_stats, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_decode_values_attend(_layer_ref(layer), batch, seq_len, q_heads, _ptr(v_codes), _ptr(v_scales),
                                            _ptr(Vhat_prev), _ptr(Khat), _ptr(scores), _ptr(Vhat), _ptr(out),
                                            _ptr(row_stats), ws, nbytes, _stream(stream)))


def aquakv_attend_raw(dtype, batch: int, tokens: int, kv_heads: int, q_heads: int, K, V, q, score_scale: float, out,
                      row_stats, accumulate: bool, stream=None, rope_cos=None, rope_sin=None) -> None:
    code = dtype if isinstance(dtype, int) else _dtype_code(dtype)
    _check(_lib.aquakv_attend_raw(code, batch, tokens, kv_heads, q_heads, _ptr(K), _ptr(V), _ptr(q), _ptr(rope_cos),
                                  _ptr(rope_sin), ctypes.c_float(score_scale), _ptr(out), _ptr(row_stats),
                                  int(bool(accumulate)), _stream(stream)))


def aquakv_fit_workspace_bytes(d_in: int, d_out: int) -> int:
    return _lib.aquakv_fit_workspace_bytes(d_in, d_out)


def aquakv_fit_predictor(dtype, tokens: int, x0, d0: int, x1, d1: int, Y, d_out: int, rate: float, W, W64, workspace,
                         stream=None, bias=None) -> None:
    """dtype: torch.bfloat16 / torch.float32 (or the C enum value).  bias: fp32 [d_out] out, fits an intercept too."""
    ws, nbytes = _ws(workspace)
    code = dtype if isinstance(dtype, int) else _dtype_code(dtype)
    _check(_lib.aquakv_fit_predictor(code, tokens, _ptr(x0), d0, _ptr(x1), d1, _ptr(Y), d_out, ctypes.c_double(rate),
                                     _ptr(W), _ptr(W64), _ptr(bias), ws, nbytes, _stream(stream)))


def aquakv_decode_attn_scores_rope(layer, batch: int, seq_len: int, q_heads: int, k_codes, k_scales, Khat_prev, q,
                                   rope_cos, rope_sin, score_scale: float, scores, Khat_out, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_decode_attn_scores_rope(_layer_ref(layer), batch, seq_len, q_heads, _ptr(k_codes), _ptr(k_scales),
                                               _ptr(Khat_prev), _ptr(q), _ptr(rope_cos), _ptr(rope_sin),
                                               ctypes.c_float(score_scale), _ptr(scores), _ptr(Khat_out), ws, nbytes,
                                               _stream(stream)))


def aquakv_decode_attn_scores(layer, batch: int, seq_len: int, q_heads: int, k_codes, k_scales, Khat_prev, q,
                              score_scale: float, scores, Khat_out, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_decode_attn_scores(_layer_ref(layer), batch, seq_len, q_heads, _ptr(k_codes), _ptr(k_scales),
                                          _ptr(Khat_prev), _ptr(q), ctypes.c_float(score_scale), _ptr(scores),
                                          _ptr(Khat_out), ws, nbytes, _stream(stream)))


def aquakv_decode_attn_scores_folded(layer, batch: int, seq_len: int, q_heads: int, k_codes, k_scales, Khat_prev, q,
                                     score_scale: float, scores, workspace, stream=None) -> None:
    ws, nbytes = _ws(workspace)
    _check(_lib.aquakv_decode_attn_scores_folded(_layer_ref(layer), batch, seq_len, q_heads, _ptr(k_codes), _ptr(k_scales),
                                                 _ptr(Khat_prev), _ptr(q), ctypes.c_float(score_scale), _ptr(scores),
                                                 ws, nbytes, _stream(stream)))


def aquakv_decode_attn_scores_folded_static(layer, batch: int, seq_len: int, q_heads: int, k_codes, k_scales, Khat_prev,
                                            q, score_scale: float, scores, stream=None) -> None:
    _check(_lib.aquakv_decode_attn_scores_folded_static(_layer_ref(layer), batch, seq_len, q_heads, _ptr(k_codes),
                                                        _ptr(k_scales), _ptr(Khat_prev), _ptr(q),
                                                        ctypes.c_float(score_scale), _ptr(scores), _stream(stream)))
