"""Randomised property checks of the CPU oracle (hypothesis): identities that hold for every input, at shapes
and values the hand-written pins do not enumerate."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import aquakv_oracle as O

SET = dict(max_examples=40, deadline=None, derandomize=True, database=None)     # the same examples on every run


def arrays(seed, shape, scale=1.0):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape) * scale


@settings(**SET)
@given(seed=st.integers(0, 2**31), n=st.sampled_from([4, 16, 64, 256]), groups=st.integers(1, 5), g=st.sampled_from([8, 16, 128]))
def test_pack_unpack_round_trip_and_size(seed, n, groups, g):
    idx = np.random.Generator(np.random.PCG64(seed)).integers(0, n, size=(groups, g // 2))
    packed = O.pack_codes(idx, n)
    assert packed.dtype == np.uint8 and packed.shape == (groups, (g // 2) * O.code_bits(n) // 8)
    assert np.array_equal(O.unpack_codes(packed, n), idx)
    # little-endian bit string: code i sits at bits [i c, (i + 1) c) of the group's bytes read as one integer
    c = O.code_bits(n)
    for row, codes in zip(packed, idx):
        big = int.from_bytes(row.tobytes(), "little")
        assert all((big >> (i * c)) & (n - 1) == int(v) for i, v in enumerate(codes))


@settings(**SET)
@given(seed=st.integers(0, 2**31), g=st.sampled_from([2, 16, 128, 1024]), rows=st.integers(1, 4), scale=st.floats(1e-3, 1e3))
def test_rht_is_an_isometry_with_the_stated_inverse(seed, g, rows, scale):
    r = arrays(seed, (rows, g), scale)
    s = np.where(arrays(seed + 1, (g,)) < 0, -1, 1).astype(np.int8)
    z = O.rht(r, s)
    assert np.allclose(np.sum(z * z, axis=-1), np.sum(r * r, axis=-1), rtol=1e-12)
    assert np.allclose(O.irht(z, s), r, rtol=1e-12, atol=1e-12 * scale)
    # linear: the transform of a sum is the sum of the transforms
    r2 = arrays(seed + 2, (rows, g), scale)
    assert np.allclose(O.rht(r + 2 * r2, s), z + 2 * O.rht(r2, s), rtol=1e-12, atol=1e-12 * scale)


@settings(**SET)
@given(seed=st.integers(0, 2**31), n=st.sampled_from([4, 16, 64]), m=st.integers(1, 50))
def test_nearest_codeword_is_never_beaten(seed, n, m):
    C = arrays(seed, (n, 2))
    y = arrays(seed + 1, (m, 2), 1.5)
    idx, gap = O.nearest_codeword(y, C)
    assert np.all(gap >= 0)
    d = np.sum((y[:, None, :] - C[None, :, :]) ** 2, axis=-1)
    assert np.all(d[np.arange(m), idx] <= d.min(axis=1))
    # lowest index among the minimisers
    assert np.array_equal(idx, np.argmin(d, axis=1))


@settings(**SET)
@given(seed=st.integers(0, 2**31), bits=st.sampled_from([2, 4]), groups=st.integers(1, 6), scale=st.floats(1e-2, 1e2),
       shift=st.floats(-3, 3))
def test_round_to_nearest_error_is_at_most_half_a_step_and_zero_is_a_level(seed, bits, groups, scale, shift):
    r = (arrays(seed, (groups * 64,)) + shift) * scale
    codes, step16, zero, _ = O.rtn_quantize(r, bits)
    assert codes.shape == (groups, 64) and step16.shape == zero.shape == (groups,)
    rec = O.rtn_dequantize(codes, step16, zero).reshape(groups, 64)
    x = r.reshape(groups, 64)
    step = step16.astype(np.float64)[:, None]
    L = (1 << bits) - 1
    # values inside the representable range [-zero, L - zero] * step are off by at most half a step
    inside = (x >= -zero[:, None] * step) & (x <= (L - zero[:, None]) * step)
    assert np.all(np.abs(rec - x)[inside] <= (0.5 * step * np.ones_like(x))[inside] * (1 + 1e-12))
    assert codes.min() >= 0 and codes.max() <= L
    # the zero point is a level: code = zero decodes to exactly 0
    zeros = O.rtn_dequantize(zero[:, None] * np.ones((groups, 64), dtype=np.int64), step16, zero)
    assert np.all(zeros == 0.0)


@settings(**SET)
@given(seed=st.integers(0, 2**31), rows=st.integers(1, 6), n=st.integers(1, 40), shift=st.floats(-500, 500))
def test_softmax_rows_are_distributions_and_ignore_a_shift(seed, rows, n, shift):
    s = arrays(seed, (rows, n), 6.0)
    p = O.softmax_rows(s)
    assert np.all(p >= 0) and np.allclose(p.sum(axis=-1), 1.0, atol=1e-14)
    assert np.allclose(O.softmax_rows(s + shift), p, rtol=1e-9, atol=1e-300)
    assert np.array_equal(np.argmax(p, axis=-1), np.argmax(s, axis=-1))


@settings(**SET)
@given(seed=st.integers(0, 2**31), tokens=st.integers(2, 12), split=st.integers(1, 11), rep=st.sampled_from([1, 2, 4]))
def test_attention_over_a_union_is_the_merge_of_its_parts(seed, tokens, split, rep):
    split = min(split, tokens - 1)
    H, g, Bn = 2, 8, 2
    q = arrays(seed, (Bn, H * rep, g))
    K, V = arrays(seed + 1, (2, Bn, tokens, H, g))
    out, M, L = O.attention(q, K, V, 0.7)
    oa, Ma, La = O.attention(q, K[:, :split], V[:, :split], 0.7)
    ob, Mb, Lb = O.attention(q, K[:, split:], V[:, split:], 0.7)
    Mm = np.maximum(Ma, Mb)
    wa, wb = La * np.exp(Ma - Mm), Lb * np.exp(Mb - Mm)
    assert np.allclose(Mm, M) and np.allclose(wa + wb, L, rtol=1e-12)
    assert np.allclose((oa * wa[..., None] + ob * wb[..., None]) / (wa + wb)[..., None], out, rtol=1e-11, atol=1e-13)
