"""GPU parity for the second backbone of Sect. 4.1 of the AQUA-KV paper (uniform round-to-nearest, groups of 64):
the HIP library through its C ABI against the CPU oracle.  Codes, steps and zero points bit-exact except counted
rounding ties; reconstructions within 1e-5 (fp32) / 2e-2 (bf16) relative; decode reproduces encode bit for bit."""
import numpy as np
import pytest
import torch

from oracle import aquakv_oracle as O
from paper_2501_19392_amd import synth
from tests import parity_utils as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests must run on an MI355X")
    from paper_2501_19392_amd import binding
    return binding


def storage_randn(shape, dtype, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(*shape, generator=g) * scale).to(synth.torch_dtype(dtype)).cuda()


def bits_of(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


@pytest.mark.parametrize("dtype,bits,T,H", [("fp32", 2, 256, 2), ("bf16", 2, 300, 8), ("bf16", 4, 257, 8), ("fp32", 4, 33, 1)])
@pytest.mark.parametrize("with_p", [False, True])
def test_rtn_quantize_stage(B, dtype, bits, T, H, with_p):
    print(f"case rtn quantize dtype={dtype} bits={bits} T={T} H={H} with_p={with_p}", flush=True)
    lo, lg = U.make_layers(H, dtype, None, rtn_bits=bits)
    D = H * 128
    ch = synth.channel_scales(D, 0, 0).float()
    g = torch.Generator().manual_seed(70)
    X = (torch.randn(T, D, generator=g) * ch).to(synth.torch_dtype(dtype)).cuda().reshape(T, H, 128)
    P = (storage_randn((T, D), "fp32", 71) * 0.8).reshape(T, H, 128).contiguous() if with_p else None
    codes, meta = lg.alloc_codes(T)
    assert codes.shape == (T, H, 16 * bits) and meta.shape == (T, D // 64, 2)
    Xhat = lg.alloc_kv(T)
    B.aquakv_quantize(lg, B.AQUAKV_KEY, T, X, P, codes, meta, Xhat)
    torch.cuda.synchronize()
    p64 = np.zeros((T, D)) if P is None else U.np64(P).reshape(T, D)
    rep = U.compare_rtn_outputs(U.np64(X).reshape(T, D) - p64, codes.cpu().numpy(), meta.cpu().numpy(), bits)
    print("  ", rep, flush=True)
    assert rep.other == 0, str(rep)
    assert rep.code_mismatch <= max(2, rep.subvectors // 20000) and rep.scale_mismatch <= max(1, rep.groups // 500)
    # the reconstruction is the oracle's decode of the GPU's own codes, and what the dequantize entry point gives
    want = O.round_storage(U.rtn_decode(codes.cpu().numpy(), meta.cpu().numpy(), bits, T) + p64, dtype)
    U.assert_close_storage(Xhat, want.reshape(T, H, 128), dtype, "Xhat")
    X2 = lg.alloc_kv(T)
    B.aquakv_dequantize(lg, B.AQUAKV_KEY, T, codes, meta, P, X2)
    torch.cuda.synchronize()
    assert torch.equal(bits_of(X2), bits_of(Xhat))


def test_rtn_edge_groups(B):
    """All-zero group, constant groups of either sign, a group beyond the fp16 range of the step, one token."""
    print("case rtn edge groups", flush=True)
    H, T = 2, 5
    lo, lg = U.make_layers(H, "fp32", None, rtn_bits=2)
    X = torch.zeros(T, H * 128)
    X[1, :64] = 2.5
    X[1, 64:128] = -1.25
    X[2] = torch.randn(H * 128, generator=torch.Generator().manual_seed(72)) * 1e6     # step clamps to 65504
    X[3] = torch.randn(H * 128, generator=torch.Generator().manual_seed(73)) * 1e-7    # step underflows fp16 towards 0
    X[4] = torch.randn(H * 128, generator=torch.Generator().manual_seed(74))
    Xg = X.cuda().reshape(T, H, 128)
    codes, meta = lg.alloc_codes(T)
    Xhat = lg.alloc_kv(T)
    B.aquakv_quantize(lg, B.AQUAKV_VALUE, T, Xg, None, codes, meta, Xhat)
    torch.cuda.synchronize()
    rep = U.compare_rtn_outputs(U.np64(X), codes.cpu().numpy(), meta.cpu().numpy(), 2)
    print("  ", rep, flush=True)
    assert rep.other == 0 and rep.code_mismatch == 0 and rep.scale_mismatch == 0, str(rep)
    assert not Xhat[0].any() and not codes[0].any() and not meta[0].any()
    # constant groups: every value takes the top (or bottom) code; off only by the fp16 rounding of the step
    assert torch.allclose(Xhat[1].reshape(-1)[:128], X[1, :128].cuda(), rtol=2 ** -11, atol=0)
    want = O.round_storage(U.rtn_decode(codes.cpu().numpy(), meta.cpu().numpy(), 2, T), "fp32")
    U.assert_close_storage(Xhat, want.reshape(T, H, 128), "fp32", "edge Xhat")
    # one token, and none
    c1, m1 = lg.alloc_codes(1)
    B.aquakv_quantize(lg, B.AQUAKV_VALUE, 1, Xg[4:5].contiguous(), None, c1, m1, None)
    B.aquakv_quantize(lg, B.AQUAKV_VALUE, 0, Xg, None, codes, meta, None)
    torch.cuda.synchronize()
    assert torch.equal(c1[0], codes[4]) and torch.equal(m1[0], meta[4])


@pytest.mark.parametrize("dtype,bits,T", [("bf16", 2, 515), ("fp32", 2, 200), ("bf16", 4, 300)])
def test_rtn_layer_stack(B, dtype, bits, T):
    """Three layers with predictors (bf16: the fused kernels; fp32: predictor and quantizer apart): every stage
    teacher-forced against the oracle, decode bit-identical to encode, the scoring call against the definition,
    the key / value halves identical to the layer call."""
    print(f"case rtn stack dtype={dtype} bits={bits} T={T}", flush=True)
    H, QH = 8, 16
    D = H * 128
    cfg = synth.Config("rtn-test", layers=3, kv_heads=H, head_dim=128, tokens=T, dtype=dtype)
    st = synth.KVStream(cfg, device="cpu", work=torch.float64)
    layers, Ks, Vs = [], [], []
    for l in range(3):
        K, V = st.next()
        Ks.append(K.cuda()); Vs.append(V.cuda())
        if l == 0:
            layers.append(U.make_layers(H, dtype, None, rtn_bits=bits))
        else:
            wk, wv = synth.analytic_predictors(st, l)
            gb = torch.Generator().manual_seed(80 + l)
            layers.append(U.make_layers(H, dtype, None, w_k=wk, w_v=wv, b_k=torch.randn(D, generator=gb) * 0.2,
                                        b_v=torch.randn(D, generator=gb) * 0.2, rtn_bits=bits))
    Kp = Vp = None
    outs = []
    for l, (lo, lg) in enumerate(layers):
        kc, km = lg.alloc_codes(T)
        vc, vm = lg.alloc_codes(T)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        ws = lg.alloc_workspace(T)
        B.aquakv_encode_layer(lg, T, Ks[l], Vs[l], Kp, Vp, kc, km, vc, vm, Kh, Vh, ws)
        torch.cuda.synchronize()
        # stage by stage, on the GPU's own inputs
        for which, X, codes, meta, hat in (("k", Ks[l], kc, km, Kh), ("v", Vs[l], vc, vm, Vh)):
            if l == 0:
                p64 = np.zeros((T, D))
            else:
                P = torch.empty(T, D, dtype=torch.float32, device="cuda")
                if which == "k":
                    B.aquakv_predict(lg, B.AQUAKV_KEY, T, Kp, None, P)
                    xin, W, b = U.np64(Kp).reshape(T, D), lo.w_k, lo.b_k
                else:
                    B.aquakv_predict(lg, B.AQUAKV_VALUE, T, Vp, Kh, P)
                    xin, W, b = np.concatenate([U.np64(Vp).reshape(T, D), U.np64(Kh).reshape(T, D)], 1), lo.w_v, lo.b_v
                torch.cuda.synchronize()
                p64 = U.np64(P)
                assert np.all(np.abs(p64 - O.predict(xin, W, b)) <= 4e-6 * (np.abs(xin) @ np.abs(W).T + np.abs(b)) + 1e-30)
            rep = U.compare_rtn_outputs(U.np64(X).reshape(T, D) - p64, codes.cpu().numpy(), meta.cpu().numpy(), bits)
            print(f"   layer {l} {which}: {rep}", flush=True)
            assert rep.other == 0, str(rep)
            assert rep.code_mismatch <= max(2, rep.subvectors // 20000) and rep.scale_mismatch <= max(1, rep.groups // 500)
            want = O.round_storage(U.rtn_decode(codes.cpu().numpy(), meta.cpu().numpy(), bits, T) + p64, dtype)
            U.assert_close_storage(hat, want.reshape(T, H, 128), dtype, which + "hat")
        # decode reproduces encode bit for bit
        Kd, Vd = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_decode_layer(lg, T, kc, km, vc, vm, Kp, Vp, Kd, Vd, ws)
        torch.cuda.synchronize()
        assert torch.equal(bits_of(Kd), bits_of(Kh)) and torch.equal(bits_of(Vd), bits_of(Vh))
        # the halves give the same bits as the layer call
        kc2, km2 = lg.alloc_codes(T)
        vc2, vm2 = lg.alloc_codes(T)
        Kh2, Vh2 = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_encode_keys(lg, T, Ks[l], Kp, kc2, km2, Kh2, ws)
        B.aquakv_encode_values(lg, T, Vs[l], Vp, Kh2, vc2, vm2, Vh2, ws)
        torch.cuda.synchronize()
        assert torch.equal(kc2, kc) and torch.equal(km2, km) and torch.equal(vc2, vc) and torch.equal(vm2, vm)
        assert torch.equal(bits_of(Kh2), bits_of(Kh)) and torch.equal(bits_of(Vh2), bits_of(Vh))
        # scores from the codes: q . Khat, with the reconstruction as a by-product
        q = storage_randn((1, QH, 128), dtype, 90 + l)
        scores = torch.empty(1, QH, T, dtype=torch.float32, device="cuda")
        Ko = lg.alloc_kv(T)
        B.aquakv_decode_attn_scores(lg, 1, T, QH, kc, km, Kp, q, 0.25, scores, Ko, ws)
        torch.cuda.synchronize()
        assert torch.equal(bits_of(Ko), bits_of(Kh))
        want = 0.25 * np.einsum("qd,tqd->qt", U.np64(q)[0], np.repeat(U.np64(Kh), QH // H, axis=1))
        mag = 0.25 * np.einsum("qd,tqd->qt", np.abs(U.np64(q)[0]), np.repeat(np.abs(U.np64(Kh)), QH // H, axis=1))
        assert np.all(np.abs(U.np64(scores)[0] - want) <= 4e-6 * mag + 1e-30)
        # without the by-product: layers with a key predictor take the folded form in bf16 (predictor folded into the
        # query, code term step * sum q (code - zero) per group), everything else recomputes as above
        s2 = torch.full_like(scores, float("nan"))
        folded = l > 0 and dtype == "bf16"
        assert (B.aquakv_scores_workspace_bytes(lg, 1, QH) > 0) == folded
        if folded:
            B.aquakv_decode_attn_scores_folded(lg, 1, T, QH, kc, km, Kp, q, 0.25, s2, lg.alloc_scores_workspace(1, QH))
        else:
            B.aquakv_decode_attn_scores(lg, 1, T, QH, kc, km, Kp, q, 0.25, s2, None, ws)
        torch.cuda.synchronize()
        if folded:
            worst = float(np.max(np.abs(U.np64(s2)[0] - want) / (mag + 1e-30)))
            print(f"   layer {l}: folded scores, worst error / (sum|q||k|) = {worst:.3g}", flush=True)
            assert np.all(np.abs(U.np64(s2)[0] - want) <= U.RTOL["bf16"] * mag + 1e-30), worst
            assert not torch.equal(s2, scores)                 # (it really is another path)
            # this backbone has neither rotation nor grid: whatever a C caller left in those fields of the struct
            # (here: a sign vector of -1s, misaligned grid and table pointers) is ignored, also by the folded form
            junk = torch.full((2048,), -1, dtype=torch.int8, device="cuda")
            c2 = B.aquakv_layer.from_buffer_copy(lg.c)
            c2.signs_k, c2.signs_v = junk.data_ptr(), junk.data_ptr() + 1024
            c2.codebook, c2.search_table = junk.data_ptr() + 4, junk.data_ptr() + 8
            s3 = torch.full_like(scores, float("nan"))
            B.aquakv_decode_attn_scores_folded(c2, 1, T, QH, kc, km, Kp, q, 0.25, s3, lg.alloc_scores_workspace(1, QH))
            s4 = torch.full_like(scores, float("nan"))
            B.aquakv_decode_attn_scores(c2, 1, T, QH, kc, km, Kp, q, 0.25, s4, None, ws)
            torch.cuda.synchronize()
            assert torch.equal(s3, s2) and torch.equal(s4, scores)
        else:
            assert torch.equal(s2, scores)
        outs.append((kc, km, vc, vm))
        Kp, Vp = Kh, Vh
    # the free-running oracle (no teacher forcing) stays close: same codes wherever no rounding tie moved one
    Kp = Vp = None
    for l, (lo, lg) in enumerate(layers):
        e = O.encode_layer(lo, U.np64(Ks[l]), U.np64(Vs[l]), Kp, Vp)
        frac = float(np.mean(e["k_codes"].reshape(T, -1) != outs[l][0].cpu().numpy().reshape(T, -1)))
        print(f"   free-run layer {l}: key code bytes differing {frac:.2e}", flush=True)
        assert frac < (2e-2 if dtype == "bf16" else 1e-3)
        Kp, Vp = e["Khat"], e["Vhat"]


@pytest.mark.parametrize("dtype,bits", [("bf16", 2), ("fp32", 4)])
def test_rtn_groups_of_1024(B, dtype, bits):
    """Groups of 1024 = the whole token of 8 heads, one (step, zero) per token (2 + 32 / 1024 = 2.03 stored bits at
    2 bits, the appendix table of Sect. 4.1): every stage against the oracle, closed loop, scores."""
    print(f"case rtn groups of 1024 dtype={dtype} bits={bits}", flush=True)
    H, T, QH = 8, 203, 16
    D = H * 128
    cfg = synth.Config("rtn-1024", layers=2, kv_heads=H, head_dim=128, tokens=T, dtype=dtype)
    st = synth.KVStream(cfg, device="cpu", work=torch.float64)
    K0, V0 = (t.cuda() for t in st.next())
    K1, V1 = (t.cuda() for t in st.next())
    wk, wv = synth.analytic_predictors(st, 1)
    lo0, lg0 = U.make_layers(H, dtype, None, rtn_bits=bits, rht_group=1024)
    lo1, lg1 = U.make_layers(H, dtype, None, w_k=wk, w_v=wv, rtn_bits=bits, rht_group=1024)
    Kp = Vp = None
    for l, (lo, lg, K, V) in enumerate(((lo0, lg0, K0, V0), (lo1, lg1, K1, V1))):
        kc, km = lg.alloc_codes(T)
        vc, vm = lg.alloc_codes(T)
        assert km.shape == (T, 1, 2)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        ws = lg.alloc_workspace(T)
        B.aquakv_encode_layer(lg, T, K, V, Kp, Vp, kc, km, vc, vm, Kh, Vh, ws)
        torch.cuda.synchronize()
        for which, X, codes, meta, hat in (("k", K, kc, km, Kh), ("v", V, vc, vm, Vh)):
            if l == 0:
                p64 = np.zeros((T, D))
            else:
                P = torch.empty(T, D, dtype=torch.float32, device="cuda")
                if which == "k":
                    B.aquakv_predict(lg, B.AQUAKV_KEY, T, Kp, None, P)
                else:
                    B.aquakv_predict(lg, B.AQUAKV_VALUE, T, Vp, Kh, P)
                torch.cuda.synchronize()
                p64 = U.np64(P)
            rep = U.compare_rtn_outputs(U.np64(X).reshape(T, D) - p64, codes.cpu().numpy(), meta.cpu().numpy(), bits, group=1024)
            print(f"   layer {l} {which}: {rep}", flush=True)
            assert rep.other == 0 and rep.groups == T, str(rep)
            idx = O.unpack_codes(codes.cpu().numpy().reshape(T, 1, -1), 1 << bits)
            s16, zero = O.rtn_unpack_meta(meta.cpu().numpy().reshape(T, 1, 2))
            want = O.round_storage(O.rtn_dequantize(idx, s16, zero) + p64, dtype)
            U.assert_close_storage(hat, want.reshape(T, H, 128), dtype, which + "hat")
        stored_bits = 8.0 * (kc[0].numel() + km[0].numel() * 2) / D
        assert abs(stored_bits - (bits + 32 / 1024)) < 1e-12
        Kd, Vd = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_decode_layer(lg, T, kc, km, vc, vm, Kp, Vp, Kd, Vd, ws)
        q = storage_randn((1, QH, 128), dtype, 95 + l)
        scores = torch.empty(1, QH, T, dtype=torch.float32, device="cuda")
        B.aquakv_decode_attn_scores(lg, 1, T, QH, kc, km, Kp, q, 0.5, scores, None, ws)
        torch.cuda.synchronize()
        assert torch.equal(bits_of(Kd), bits_of(Kh)) and torch.equal(bits_of(Vd), bits_of(Vh))
        k64 = np.repeat(U.np64(Kh), QH // H, axis=1)
        want = 0.5 * np.einsum("qd,tqd->qt", U.np64(q)[0], k64)
        mag = 0.5 * np.einsum("qd,tqd->qt", np.abs(U.np64(q)[0]), np.abs(k64))
        assert np.all(np.abs(U.np64(scores)[0] - want) <= 4e-6 * mag + 1e-30)
        Kp, Vp = Kh, Vh
