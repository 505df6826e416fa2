"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2501_19392_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a 16-byte aligned non-NULL address; never dereferenced on a validation error


def header_symbols():
    text = open(os.path.join(ROOT, "include", "aquakv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aquakv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = header_symbols()
    assert set(syms) == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for s in syms:
        assert hasattr(lib, s), s
    assert B.aquakv_version() == 100
    assert B.aquakv_status_string(0) == "ok" and "workspace" in B.aquakv_status_string(B.AQUAKV_EWORKSPACE)


def layer(**kw):
    d = dict(kv_heads=8, head_dim=128, vq_dim=2, n_codewords=16, dtype=B.AQUAKV_BF16, d_in_k=1024, d_in_v=2048,
             rht_group=0, codebook=FAKE, signs_k=FAKE, signs_v=FAKE, w_k=FAKE, b_k=None, w_v=FAKE, b_v=None,
             search_table=None)
    d.update(kw)
    return B.aquakv_layer(**d)


def status_of(fn, *a):
    with pytest.raises(B.AquaKVError) as e:
        fn(*a)
    return e.value.status


ENC_OK = [FAKE] * 10  # K V Khat_prev Vhat_prev k_codes k_scales v_codes v_scales Khat Vhat


@pytest.mark.parametrize("kw,want", [
    (dict(head_dim=100), B.AQUAKV_EINVAL),
    (dict(head_dim=64), B.AQUAKV_EUNSUPPORTED),
    (dict(vq_dim=4), B.AQUAKV_EUNSUPPORTED),
    (dict(n_codewords=17), B.AQUAKV_EINVAL),
    (dict(n_codewords=32), B.AQUAKV_EUNSUPPORTED),
    (dict(dtype=7), B.AQUAKV_EINVAL),
    (dict(kv_heads=0), B.AQUAKV_EINVAL),
    (dict(d_in_k=100), B.AQUAKV_EINVAL),
    (dict(d_in_v=1024), B.AQUAKV_EINVAL),
    (dict(codebook=None), B.AQUAKV_ENULL),
    (dict(w_k=None), B.AQUAKV_ENULL),
    (dict(signs_v=FAKE + 4), B.AQUAKV_EALIGN),
    (dict(rht_group=64), B.AQUAKV_EINVAL),
    (dict(rht_group=512, kv_heads=4, d_in_v=1024), B.AQUAKV_EUNSUPPORTED),
])
def test_bad_layer_is_rejected(kw, want):
    L = layer(**kw)
    assert status_of(B.aquakv_encode_layer, L, 128, *ENC_OK, (FAKE, 1 << 40)) == want
    assert B.aquakv_workspace_bytes(L, 128) == 0
    assert B.aquakv_last_error() != ""


def test_decode_tile_rule():
    """The 256 x two-head tile is taken when it costs no extra round of workgroups over 256 compute units (one
    workgroup per CU at a time): with 8 kv heads a row tile is 4 large or 8 small workgroups."""
    L = layer()
    rounds = lambda wgs: -(-wgs // 256)
    for T in (1, 256, 8192, 8193, 16384, 16385, 24576, 24577, 32768, 40000, 65536, 1 << 20):
        big = -(-min(T, 65536) // 256) * 4                    # calls are cut into chunks of 65536 rows
        want = 2 if 2 * rounds(big) <= rounds(2 * big) else 1
        assert B.aquakv_fused_tile_heads(L, T) == want, T
    assert [B.aquakv_fused_tile_heads(L, T) for T in (8192, 8193, 16384, 16385, 32768)] == [1, 2, 2, 1, 2]
    assert B.aquakv_fused_tile_heads(layer(kv_heads=3, d_in_k=384, d_in_v=768), 32768) == 1      # D not a multiple of 256
    assert B.aquakv_fused_tile_heads(layer(rht_group=1024), 32768) == 2                           # groups across the heads: the decode kernels' tile
    assert B.aquakv_fused_tile_heads(layer(dtype=B.AQUAKV_FP32), 32768) == 0                      # separate kernels
    assert B.aquakv_fused_tile_heads(layer(d_in_k=0, d_in_v=0, w_k=None, w_v=None), 32768) == 0   # no predictor
    assert B.aquakv_fused_tile_heads(L, 0) == 0 and B.aquakv_fused_tile_heads(layer(head_dim=64), 32768) == 0


def test_bad_call_arguments_are_rejected_without_launching():
    L = layer()
    need = B.aquakv_workspace_bytes(L, 300)
    assert need == 300 * 1024 * 2                                            # bf16: only a temporary Khat
    assert B.aquakv_workspace_bytes(L, 1 << 20) == 65536 * 1024 * 2          # chunked: bounded
    L32 = layer(dtype=B.AQUAKV_FP32)
    assert B.aquakv_workspace_bytes(L32, 300) == 300 * 1024 * (4 + 4)        # fp32: predictions + Khat
    assert B.aquakv_workspace_bytes(L32, 1 << 20) == 16384 * 1024 * 8
    Lw = layer(rht_group=1024)                 # groups across heads: the larger predictor's weights re-tiled + a temporary Khat
    assert B.aquakv_workspace_bytes(Lw, 300) == 1024 * 2048 * 2 + 300 * 1024 * 2
    args = list(ENC_OK)
    assert status_of(B.aquakv_encode_layer, L, -1, *args, (FAKE, need)) == B.AQUAKV_EINVAL
    assert status_of(B.aquakv_encode_layer, L, 300, *args, (FAKE, need - 1)) == B.AQUAKV_EWORKSPACE
    assert "workspace" in B.aquakv_last_error()
    assert status_of(B.aquakv_encode_layer, L, 300, *args, None) == B.AQUAKV_ENULL
    for i in (0, 1, 2, 3, 4, 5, 6, 7):                                          # required pointers
        bad = list(args)
        bad[i] = None
        assert status_of(B.aquakv_encode_layer, L, 300, *bad, (FAKE, need)) == B.AQUAKV_ENULL
        bad[i] = FAKE + (1 if i in (5, 7) else 8)        # scale arrays need 2-byte alignment, the rest 16
        assert status_of(B.aquakv_encode_layer, L, 300, *bad, (FAKE, need)) == B.AQUAKV_EALIGN
    # tokens == 0 is a no-op even without a workspace
    B.aquakv_encode_layer(L, 0, *args, None)
    B.aquakv_decode_layer(L, 0, *([FAKE] * 8), None)
    # layer 0 (no predictors) needs no *_prev
    L0 = layer(d_in_k=0, d_in_v=0, w_k=None, w_v=None)
    a0 = list(args)
    a0[2] = a0[3] = None
    assert status_of(B.aquakv_encode_layer, L0, 300, *a0, (FAKE, 10)) == B.AQUAKV_EWORKSPACE
    # stage calls
    assert status_of(B.aquakv_predict, L0, B.AQUAKV_KEY, 8, FAKE, None, FAKE) == B.AQUAKV_EINVAL
    assert status_of(B.aquakv_predict, L, B.AQUAKV_VALUE, 8, FAKE, None, FAKE) == B.AQUAKV_ENULL
    assert status_of(B.aquakv_predict, L, 5, 8, FAKE, FAKE, FAKE) == B.AQUAKV_EINVAL
    assert status_of(B.aquakv_quantize, L, B.AQUAKV_KEY, 8, FAKE, None, None, FAKE, None) == B.AQUAKV_ENULL
    assert status_of(B.aquakv_dequantize, L, B.AQUAKV_KEY, 8, FAKE, FAKE, None, None) == B.AQUAKV_ENULL
    # search table
    assert B.aquakv_search_table_bytes(16) == (64 * 64 + 2 * 128) * 4 and B.aquakv_search_table_bytes(17) == 0
    assert status_of(B.aquakv_build_search_table, FAKE, 2, 16, None) == B.AQUAKV_ENULL
    assert status_of(B.aquakv_build_search_table, FAKE, 2, 48, FAKE) == B.AQUAKV_EINVAL
    assert status_of(B.aquakv_build_search_table, FAKE, 3, 16, FAKE) == B.AQUAKV_EUNSUPPORTED
    # scores
    sc = [FAKE, FAKE, FAKE, FAKE, 1.0, FAKE, None]
    assert status_of(B.aquakv_decode_attn_scores, L, 2, 16, 12, *sc, (FAKE, 1 << 30)) == B.AQUAKV_EINVAL   # 12 % 8
    assert status_of(B.aquakv_decode_attn_scores, L, 2, 16, 128, *sc, (FAKE, 1 << 30)) == B.AQUAKV_EINVAL  # > 8x
    assert status_of(B.aquakv_decode_attn_scores, L32, 2, 16, 32, *sc, (FAKE, 16)) == B.AQUAKV_EWORKSPACE
    B.aquakv_decode_attn_scores(L, 0, 16, 32, *sc, None)
    # rotary form: both tables are required and must be aligned
    rp = [FAKE, FAKE, FAKE, FAKE]   # k_codes k_scales Khat_prev q
    assert status_of(B.aquakv_decode_attn_scores_rope, L, 2, 16, 32, *rp, None, FAKE, 1.0, FAKE, None, (FAKE, 1 << 30)) == B.AQUAKV_ENULL
    assert status_of(B.aquakv_decode_attn_scores_rope, L, 2, 16, 32, *rp, FAKE, FAKE + 4, 1.0, FAKE, None, (FAKE, 1 << 30)) == B.AQUAKV_EALIGN
    assert status_of(B.aquakv_decode_attn_scores_rope, L, 2, 16, 12, *rp, FAKE, FAKE, 1.0, FAKE, None, (FAKE, 1 << 30)) == B.AQUAKV_EINVAL
    B.aquakv_decode_attn_scores_rope(L, 0, 16, 32, *rp, FAKE, FAKE, 1.0, FAKE, None, None)


def test_scores_workspace_query():
    """aquakv_scores_workspace_bytes: nonzero exactly where the folded scoring form exists (bf16, 8 kv heads,
    key predictor with 1024 inputs, at most 64 query heads), linear in the batch and in the passes of 4 query
    heads per kv head."""
    L = layer()
    per_batch = 8 * 2 * 8 * 1024 + 32 * 128 * 4 + 32 * 4      # operands of W^T q, rotated queries, q . b
    assert B.aquakv_scores_workspace_bytes(L, 1, 32) == per_batch
    assert B.aquakv_scores_workspace_bytes(L, 64, 24) == 64 * per_batch
    assert per_batch % 16 == 0
    assert B.aquakv_scores_workspace_bytes(L, 1, 64) == 2 * per_batch                       # two passes
    assert B.aquakv_scores_workspace_bytes(L, 3, 40) == 6 * per_batch
    assert B.aquakv_scores_workspace_bytes(L, 1, 72) == 0                                   # more than 64 query heads
    assert B.aquakv_scores_workspace_bytes(L, 0, 32) == 0
    assert B.aquakv_scores_workspace_bytes(layer(dtype=B.AQUAKV_FP32), 1, 32) == 0
    assert B.aquakv_scores_workspace_bytes(layer(kv_heads=4), 1, 32) == 0
    assert B.aquakv_scores_workspace_bytes(layer(d_in_k=0, d_in_v=0, w_k=None, w_v=None), 1, 32) == 0   # layer 0
    assert B.aquakv_scores_workspace_bytes(layer(head_dim=64), 1, 32) == 0                  # invalid layer


def test_half_calls_validate_their_arguments():
    L = layer()
    ws = (FAKE, 1 << 30)
    assert status_of(B.aquakv_encode_keys, L, 8, None, FAKE, FAKE, FAKE, FAKE, ws) == B.AQUAKV_ENULL          # K
    assert status_of(B.aquakv_encode_keys, L, 8, FAKE, None, FAKE, FAKE, FAKE, ws) == B.AQUAKV_ENULL          # Khat_prev
    assert status_of(B.aquakv_encode_keys, L, -1, FAKE, FAKE, FAKE, FAKE, FAKE, ws) == B.AQUAKV_EINVAL
    assert status_of(B.aquakv_encode_values, L, 8, FAKE, FAKE, None, FAKE, FAKE, FAKE, ws) == B.AQUAKV_ENULL  # Khat is an input
    assert status_of(B.aquakv_encode_values, L, 8, FAKE, FAKE, FAKE + 8, FAKE, FAKE, FAKE, ws) == B.AQUAKV_EALIGN
    assert status_of(B.aquakv_decode_values, L, 8, FAKE, FAKE, FAKE, FAKE, None, ws) == B.AQUAKV_ENULL        # Vhat out
    L32 = layer(dtype=B.AQUAKV_FP32)
    assert status_of(B.aquakv_decode_values, L32, 8, FAKE, FAKE, FAKE, FAKE, FAKE, (FAKE, 16)) == B.AQUAKV_EWORKSPACE
    B.aquakv_encode_keys(L, 0, FAKE, FAKE, FAKE, FAKE, None, None)               # tokens == 0: no-op
    B.aquakv_encode_values(L, 0, FAKE, FAKE, FAKE, FAKE, FAKE, None, None)
    B.aquakv_decode_values(L, 0, FAKE, FAKE, FAKE, FAKE, FAKE, None)
    L0 = layer(d_in_k=0, d_in_v=0, w_k=None, w_v=None)                          # no predictors: no *_prev, no Khat input
    assert status_of(B.aquakv_encode_values, L0, 8, FAKE, None, None, None, FAKE, FAKE, ws) == B.AQUAKV_ENULL  # v_codes


def test_weighted_values_call_validates_its_arguments():
    """Value side of attention: argument checks and the workspace size (partial sums per 256 tokens, plus the
    fp32 prediction where the layer does not run fused)."""
    L = layer()
    ws = (FAKE, 1 << 30)
    ok = [FAKE] * 7                       # v_codes v_scales Vhat_prev Khat weights Vhat out
    call = B.aquakv_decode_values_weighted
    # per chunk of 256 tokens and query head: 128 sums and 2 soft-max statistics (each block rounded up to 256 bytes)
    assert B.aquakv_weighted_workspace_bytes(L, 1, 8192, 24) == 32 * 24 * 128 * 4 + 32 * 24 * 2 * 4
    assert B.aquakv_weighted_workspace_bytes(L, 3, 257, 8) == 3 * 2 * 8 * 128 * 4 + 512
    assert B.aquakv_weighted_workspace_bytes(L, 1, 100, 8) == 8 * 128 * 4 + 256
    L32 = layer(dtype=B.AQUAKV_FP32)
    assert B.aquakv_weighted_workspace_bytes(L32, 1, 100, 8) == 8 * 128 * 4 + 256 + 100 * 1024 * 4
    assert B.aquakv_weighted_workspace_bytes(L, 0, 100, 8) == 0
    assert B.aquakv_weighted_workspace_bytes(layer(head_dim=64), 1, 100, 8) == 0
    assert status_of(call, L, 1, 256, 12, *ok, ws) == B.AQUAKV_EINVAL                 # not a multiple of kv heads
    assert status_of(call, L, 1, 256, 72, *ok, ws) == B.AQUAKV_EINVAL                 # more than 8 per kv head
    assert status_of(call, L, -1, 256, 8, *ok, ws) == B.AQUAKV_EINVAL
    for i, name in enumerate(["v_codes", "v_scales", "Vhat_prev", "Khat", "weights", None, "out"]):
        if name is None:
            continue
        a = list(ok)
        a[i] = None
        assert status_of(call, L, 1, 256, 8, *a, ws) == B.AQUAKV_ENULL, name
    a = list(ok)
    a[4] = FAKE + 2
    assert status_of(call, L, 1, 256, 8, *a, ws) == B.AQUAKV_EALIGN
    a = list(ok)
    a[5] = None                                                                     # no Vhat: only where the sums are fused
    assert status_of(call, L, 1, 255, 8, *a, ws) == B.AQUAKV_ENULL                    # ragged sequence
    assert status_of(call, L32, 1, 256, 8, *a, ws) == B.AQUAKV_ENULL
    assert status_of(call, layer(rht_group=1024, dtype=B.AQUAKV_FP32), 1, 256, 8, *a, ws) == B.AQUAKV_ENULL
    assert status_of(call, layer(d_in_k=0, d_in_v=0, w_k=None, w_v=None), 1, 256, 8, FAKE, FAKE, None, None, FAKE, None,
                     FAKE, ws) == B.AQUAKV_ENULL                                    # first layer
    assert status_of(call, L, 1, 256, 8, *ok, (FAKE, 1024)) == B.AQUAKV_EWORKSPACE
    assert status_of(call, L, 1, 256, 8, *ok, None) == B.AQUAKV_ENULL                 # workspace
    call(L, 0, 256, 8, *ok, None)                                                   # no tokens: no-op
    call(L, 1, 0, 8, *ok, None)
    att = B.aquakv_decode_values_attend                                             # same checks, plus row_stats
    assert status_of(att, L, 1, 256, 12, *ok, None, ws) == B.AQUAKV_EINVAL
    a = list(ok)
    a[4] = None
    assert status_of(att, L, 1, 256, 8, *a, None, ws) == B.AQUAKV_ENULL               # scores
    a = list(ok)
    a[5] = None
    assert status_of(att, L32, 1, 256, 8, *a, FAKE, ws) == B.AQUAKV_ENULL             # Vhat needed
    assert status_of(att, L, 1, 256, 8, *ok, FAKE + 2, ws) == B.AQUAKV_EALIGN
    assert status_of(att, L, 1, 256, 8, *ok, None, (FAKE, 1024)) == B.AQUAKV_EWORKSPACE
    att(L, 0, 256, 8, *ok, None, None)
    assert status_of(B.aquakv_softmax, 4, 10, None, FAKE) == B.AQUAKV_ENULL
    assert status_of(B.aquakv_softmax, 4, 10, FAKE, None) == B.AQUAKV_ENULL
    assert status_of(B.aquakv_softmax, -1, 10, FAKE, FAKE) == B.AQUAKV_EINVAL
    B.aquakv_softmax(0, 10, FAKE, FAKE)
    B.aquakv_softmax(4, 0, FAKE, FAKE)
    raw = B.aquakv_attend_raw                                                       # dtype batch tokens H QH K V q scale out stats acc
    assert status_of(raw, 7, 1, 8, 8, 8, FAKE, FAKE, FAKE, 1.0, FAKE, FAKE, False) == B.AQUAKV_EINVAL
    assert status_of(raw, B.AQUAKV_BF16, 1, 8, 8, 12, FAKE, FAKE, FAKE, 1.0, FAKE, FAKE, False) == B.AQUAKV_EINVAL
    assert status_of(raw, B.AQUAKV_BF16, 1, 4097, 8, 8, FAKE, FAKE, FAKE, 1.0, FAKE, FAKE, False) == B.AQUAKV_EUNSUPPORTED
    assert status_of(raw, B.AQUAKV_BF16, 1, 8, 8, 8, None, FAKE, FAKE, 1.0, FAKE, FAKE, False) == B.AQUAKV_ENULL
    assert status_of(raw, B.AQUAKV_BF16, 1, 8, 8, 8, FAKE, FAKE, FAKE, 1.0, FAKE, None, False) == B.AQUAKV_ENULL
    assert status_of(raw, B.AQUAKV_BF16, 1, 0, 8, 8, None, None, FAKE, 1.0, FAKE, FAKE, False) == B.AQUAKV_EINVAL   # nothing to write
    raw(B.AQUAKV_BF16, 1, 0, 8, 8, None, None, FAKE, 1.0, FAKE, FAKE, True)           # nothing to merge: no-op
    raw(B.AQUAKV_BF16, 0, 8, 8, 8, FAKE, FAKE, FAKE, 1.0, FAKE, FAKE, False)


def test_round_to_nearest_backbone_layer_validation():
    """vq_dim = 1: the uniform round-to-nearest backbone (Sect. 4.1): 4 or 16 levels, groups of 64, no grid / signs,
    (step, zero point) words need 4-byte alignment."""
    rtn = dict(vq_dim=1, n_codewords=4, codebook=None, signs_k=None, signs_v=None)
    L = layer(**rtn)
    assert B.aquakv_workspace_bytes(L, 300) == 300 * 1024 * 2                # bf16: fused like the grids
    assert B.aquakv_workspace_bytes(layer(**dict(rtn, n_codewords=16, rht_group=64)), 300) == 300 * 1024 * 2
    assert B.aquakv_workspace_bytes(layer(**dict(rtn, dtype=B.AQUAKV_FP32)), 300) == 300 * 1024 * 8
    assert B.aquakv_workspace_bytes(layer(**dict(rtn, rht_group=1024)), 300) == 1024 * 2048 * 2 + 300 * 1024 * 2   # whole-token groups: + re-tiled weights
    assert B.aquakv_scores_workspace_bytes(layer(**dict(rtn, rht_group=1024)), 1, 32) == 0
    assert B.aquakv_scores_workspace_bytes(L, 1, 32) == 8 * 2 * 8 * 1024 + 32 * 128 * 4 + 32 * 4      # folded form as for the grids
    ws = (FAKE, 1 << 30)
    for kw, want in ((dict(n_codewords=8), B.AQUAKV_EUNSUPPORTED), (dict(n_codewords=5), B.AQUAKV_EINVAL),
                     (dict(n_codewords=64), B.AQUAKV_EUNSUPPORTED), (dict(rht_group=128), B.AQUAKV_EUNSUPPORTED),
                     (dict(rht_group=512), B.AQUAKV_EUNSUPPORTED), (dict(rht_group=1024, kv_heads=4, d_in_v=1024), B.AQUAKV_EUNSUPPORTED)):
        assert status_of(B.aquakv_encode_layer, layer(**dict(rtn, **kw)), 8, *ENC_OK, ws) == want, kw
    bad = list(ENC_OK)
    bad[5] = FAKE + 2                                                          # k_scales: 2-byte aligned is not enough
    assert status_of(B.aquakv_encode_layer, L, 8, *bad, ws) == B.AQUAKV_EALIGN
    bad[5] = FAKE + 4
    bad[0] = None
    assert status_of(B.aquakv_encode_layer, L, 8, *bad, ws) == B.AQUAKV_ENULL   # alignment passed, K is missing
    B.aquakv_encode_layer(L, 0, *ENC_OK, None)


def test_fit_predictor_validates_its_arguments():
    assert B.aquakv_fit_workspace_bytes(1024, 1024) == (1024 * 1024 * 2 + 2048) * 8 + 16
    assert B.aquakv_fit_workspace_bytes(2048, 1024) == (2048 * 2048 + 2048 * 1024 + 3072) * 8 + 16
    assert B.aquakv_fit_workspace_bytes(100, 1024) == 0 and B.aquakv_fit_workspace_bytes(1024, 16384) == 0
    ws = (FAKE, 1 << 40)
    ok = dict(dtype=B.AQUAKV_BF16, tokens=100, x0=FAKE, d0=1024, x1=FAKE, d1=1024, Y=FAKE, d_out=1024, rate=1e-3, W=FAKE, W64=None)
    call = lambda **kw: status_of(lambda: B.aquakv_fit_predictor(*{**ok, **kw}.values(), ws))
    assert call(dtype=5) == B.AQUAKV_EINVAL
    assert call(tokens=0) == B.AQUAKV_EINVAL
    assert call(d0=1000) == B.AQUAKV_EINVAL and call(d1=32) == B.AQUAKV_EINVAL and call(d_out=0) == B.AQUAKV_EINVAL
    assert call(d0=8192, d1=64) == B.AQUAKV_EUNSUPPORTED
    assert call(rate=-1.0) == B.AQUAKV_EINVAL and call(rate=float("nan")) == B.AQUAKV_EINVAL
    assert call(x0=None) == B.AQUAKV_ENULL and call(x1=None) == B.AQUAKV_ENULL and call(W=None) == B.AQUAKV_ENULL
    assert call(Y=FAKE + 8) == B.AQUAKV_EALIGN
    assert status_of(lambda: B.aquakv_fit_predictor(*ok.values(), (FAKE, 100))) == B.AQUAKV_EWORKSPACE
    assert status_of(lambda: B.aquakv_fit_predictor(*{**ok, "x1": None, "d1": 0}.values(), None)) == B.AQUAKV_ENULL   # x1 optional, workspace not


def test_overlapping_buffers_are_refused_before_any_launch():
    """Aliasing contract of the layer calls: an output may coincide with the tensor it reconstructs (Khat with K,
    Vhat with V); any other overlap of an output or the workspace with an input or another output is a race
    between workgroups and is refused (every case here is one, so nothing is ever launched)."""
    L = layer()
    T = 300
    row, crow, srow = 1024 * 2, 8 * 32, 8 * 2
    base = 0x10000000
    names = ["K", "V", "Khat_prev", "Vhat_prev", "k_codes", "k_scales", "v_codes", "v_scales", "Khat", "Vhat"]
    addr = {n: base + i * 0x1000000 for i, n in enumerate(names)}          # 16 MiB apart: disjoint for 300 rows
    ws = (base + 0x20000000, B.aquakv_workspace_bytes(L, T))

    def enc(ws_=ws, **kw):
        a = dict(addr)
        a.update(kw)
        with pytest.raises(B.AquaKVError) as e:
            B.aquakv_encode_layer(L, T, *[a[n] for n in names], ws_)
        assert e.value.status == B.AQUAKV_EINVAL, str(e.value)
        return str(e.value)

    assert "Vhat overlaps Vhat_prev" in enc(Vhat=addr["Vhat_prev"])
    assert "Khat overlaps Khat_prev" in enc(Khat=addr["Khat_prev"])
    assert "Khat overlaps Vhat" in enc(Vhat=addr["Khat"])
    assert "Khat overlaps K" in enc(Khat=addr["K"] + row)                 # shifted by one row: not "in place"
    assert "Vhat overlaps K" in enc(Vhat=addr["K"])                       # in place is for the tensor's own input only
    assert "Khat overlaps V" in enc(Khat=addr["V"] + (T - 1) * row)       # last row of V
    assert "k_codes overlaps v_codes" in enc(v_codes=addr["k_codes"] + (T - 1) * crow)
    assert "k_scales overlaps" in enc(k_scales=addr["K"] + 16)
    assert "workspace overlaps" in enc(ws_=(addr["Vhat_prev"] + 64, ws[1]))
    # reconstruction in place is allowed: the error below is about the codes, not about Khat / Vhat
    msg = enc(Khat=addr["K"], Vhat=addr["V"], v_codes=addr["k_codes"])
    assert "k_codes overlaps v_codes" in msg
    # just past the end is not an overlap for the buffer it follows: only the next check trips
    msg = enc(Khat=addr["K"] + T * row, Vhat=addr["Khat_prev"])
    assert "Vhat overlaps Khat_prev" in msg

    def st(fn, *a):
        with pytest.raises(B.AquaKVError) as e:
            fn(*a)
        assert e.value.status == B.AQUAKV_EINVAL, str(e.value)
        return str(e.value)

    A = addr
    assert "Khat overlaps Khat_prev" in st(B.aquakv_decode_layer, L, T, A["k_codes"], A["k_scales"], A["v_codes"], A["v_scales"],
                                           A["Khat_prev"], A["Vhat_prev"], A["Khat_prev"], A["Vhat"], ws)
    assert "Vhat overlaps v_codes" in st(B.aquakv_decode_layer, L, T, A["k_codes"], A["k_scales"], A["v_codes"], A["v_scales"],
                                         A["Khat_prev"], A["Vhat_prev"], A["Khat"], A["v_codes"], ws)
    assert "Khat overlaps Khat_prev" in st(B.aquakv_encode_keys, L, T, A["K"], A["Khat_prev"], A["k_codes"], A["k_scales"],
                                           A["Khat_prev"], ws)
    assert "Vhat overlaps Khat" in st(B.aquakv_encode_values, L, T, A["V"], A["Vhat_prev"], A["Khat"], A["v_codes"], A["v_scales"],
                                      A["Khat"], ws)
    assert "Vhat overlaps Vhat_prev" in st(B.aquakv_decode_values, L, T, A["v_codes"], A["v_scales"], A["Vhat_prev"], A["Khat"],
                                           A["Vhat_prev"], ws)
    _ = srow


def test_folded_scoring_calls_validate_their_arguments():
    """The folded form is a call of its own: EUNSUPPORTED where it is not built, its own workspace size, and the
    variant with the built-in buffer refuses shapes beyond that buffer with a text that names the other call."""
    L = layer()
    sc = [FAKE, FAKE, FAKE, FAKE, 1.0, FAKE]        # k_codes k_scales Khat_prev q scale scores
    need = B.aquakv_scores_workspace_bytes(L, 2, 32)
    f = B.aquakv_decode_attn_scores_folded
    assert status_of(f, L, 2, 16, 32, *sc, (FAKE, need - 1)) == B.AQUAKV_EWORKSPACE
    assert status_of(f, L, 2, 16, 32, *sc, None) == B.AQUAKV_ENULL
    assert status_of(f, L, 2, 16, 12, *sc, (FAKE, need)) == B.AQUAKV_EINVAL
    assert status_of(f, layer(dtype=B.AQUAKV_FP32), 2, 16, 32, *sc, (FAKE, need)) == B.AQUAKV_EUNSUPPORTED
    assert status_of(f, layer(rht_group=1024), 2, 16, 32, *sc, (FAKE, need)) == B.AQUAKV_EUNSUPPORTED
    assert status_of(f, layer(kv_heads=4, d_in_k=512, d_in_v=1024), 2, 16, 32, *sc, (FAKE, need)) == B.AQUAKV_EUNSUPPORTED
    L0 = layer(d_in_k=0, d_in_v=0, w_k=None, w_v=None)
    assert status_of(f, L0, 2, 16, 32, FAKE, FAKE, None, FAKE, 1.0, FAKE, (FAKE, need)) == B.AQUAKV_EUNSUPPORTED
    bad = list(sc)
    bad[2] = None
    assert status_of(f, L, 2, 16, 32, *bad, (FAKE, need)) == B.AQUAKV_ENULL          # Khat_prev
    f(L, 0, 16, 32, *sc, None)                                                      # no tokens: no-op
    g = B.aquakv_decode_attn_scores_folded_static
    assert status_of(g, L, 65, 16, 32, *sc) == B.AQUAKV_EUNSUPPORTED                # batch x passes > 64
    assert "aquakv_decode_attn_scores_folded" in B.aquakv_last_error()
    assert status_of(g, L, 33, 16, 64, *sc) == B.AQUAKV_EUNSUPPORTED                # two passes
    assert status_of(g, layer(head_dim=64), 1, 16, 32, *sc) == B.AQUAKV_EUNSUPPORTED  # invalid layer first


def test_round_to_nearest_backbone_ignores_grid_pointers():
    """vq_dim = 1 reads neither grid nor signs nor table: whatever the struct holds there is not even checked for alignment."""
    L = layer(vq_dim=1, n_codewords=4, codebook=FAKE + 4, signs_k=FAKE + 1, signs_v=FAKE + 2, search_table=FAKE + 8)
    assert B.aquakv_workspace_bytes(L, 300) == 300 * 1024 * 2
    B.aquakv_encode_layer(L, 0, *ENC_OK, None)
    assert status_of(B.aquakv_encode_layer, layer(vq_dim=1, n_codewords=4, w_k=FAKE + 4), 8, *ENC_OK, (FAKE, 1 << 30)) == B.AQUAKV_EALIGN
