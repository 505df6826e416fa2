"""GPU parity of the value side of attention: soft-max rows and the decode of the values with the
weighted sum over tokens, against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import aquakv_oracle as O
from paper_2501_19392_amd import synth
from tests import parity_utils as U
from tests import test_gpu_parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests must run on an MI355X")
    from paper_2501_19392_amd import binding
    return binding


def sync():
    torch.cuda.synchronize()


@pytest.mark.parametrize("rows,n", [(1, 1), (7, 5), (3, 300), (5, 4096), (24, 8192), (3, 16384), (2, 16388), (2, 20001)])
def test_softmax_rows(B, rows, n):
    print(f"case softmax rows={rows} n={n}", flush=True)
    g = torch.Generator().manual_seed(rows * 100003 + n)
    s = (torch.randn(rows, n, generator=g) * 4.0 + 30.0).cuda()
    p = torch.full_like(s, float("nan"))
    B.aquakv_softmax(rows, n, s, p)
    sync()
    want = O.softmax_rows(U.np64(s))
    got = U.np64(p)
    # fp32 exponentials and a sum of n terms: 1e-5 relative is several times what the arithmetic needs
    assert np.all(np.abs(got - want) <= 1e-5 * want + 1e-30), float(np.max(np.abs(got - want) / want))
    assert abs(got.sum(axis=1) - 1.0).max() < 1e-5
    B.aquakv_softmax(rows, n, s, s)            # in place
    sync()
    assert torch.equal(s, p)


def group_rms(Vh):
    """rms over the 128 values of every (sequence, token, head): [batch, S, H]."""
    return np.sqrt(np.mean(Vh ** 2, axis=-1))


def weights_for(batch, QH, S, seed, kind):
    g = torch.Generator().manual_seed(seed)
    if kind == "softmax":
        w = torch.softmax(torch.randn(batch, QH, S, generator=g) * 3.0, dim=-1)
    else:                                      # any real numbers, both signs, wide range
        w = torch.randn(batch, QH, S, generator=g) * torch.exp(torch.randn(batch, QH, S, generator=g))
    return w.float().cuda()


def check_weighted(B, lo, lg, g, batch, S, QH, w, fused_expected, label):
    T = batch * S
    H = lo.kv_heads
    out = torch.full((batch, QH, 128), float("nan"), dtype=torch.float32, device="cuda")
    Vout = lg.alloc_kv(T)
    ws = lg.alloc_weighted_workspace(batch, S, QH)
    B.aquakv_decode_values_weighted(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], w, Vout, out, ws)
    sync()
    assert torch.equal(P.bits(Vout), P.bits(g["Vhat"])), f"{label}: decoded values differ from the encoder's reconstruction"
    vp = None if g["Vp"] is None else U.np64(g["Vp"])
    meta = g["v_scales"].cpu().numpy()
    scales = meta if lo.rtn_bits else meta.view(np.float16)
    want, _ = O.attn_values(lo, batch, S, U.np64(w), g["v_codes"].cpu().numpy(), scales, vp, U.np64(g["Khat"]))
    # size of the sum's terms, from the GPU's own values
    Vh = U.np64(g["Vhat"]).reshape(batch, S, H, 128)
    rep = QH // H
    wa = np.abs(U.np64(w))
    mag = np.stack([np.einsum("bt,btd->bd", wa[:, qh], np.abs(Vh[:, :, qh // rep])) for qh in range(QH)], 1)
    own = np.stack([np.einsum("bt,btd->bd", U.np64(w)[:, qh], Vh[:, :, qh // rep]) for qh in range(QH)], 1)
    got = U.np64(out)
    rtol = U.RTOL[lo.dtype]
    err = np.abs(got - want)
    # the decoded values agree with the oracle's within rtol (|v| + rms of the group); the sum inherits that weight by weight
    bound = rtol * (mag + np.stack([np.einsum("bt,bt->b", wa[:, qh], group_rms(Vh)[:, :, qh // rep]) for qh in range(QH)], 1)[..., None])
    assert np.all(err <= bound + 1e-30), f"{label}: {float(np.max(err / (bound + 1e-30))):.3g}"
    # against the sum over the GPU's own decoded values the only error is the summation's: weights carried
    # with 16 mantissa bits on the matrix cores (2^-17 relative per term), fp32 accumulation otherwise
    err_own = np.abs(got - own)
    assert np.all(err_own <= 2e-5 * mag + 1e-30), f"{label}: {float(np.max(err_own / (mag + 1e-30))):.3g}"
    print(f"   {label}: worst error / sum|w||v| = {float(np.max(err / (mag + 1e-30))):.3g} against the oracle, "
          f"{float(np.max(err_own / (mag + 1e-30))):.3g} against the sum over the decoded values", flush=True)
    if fused_expected:
        out2 = torch.full_like(out, float("nan"))
        B.aquakv_decode_values_weighted(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], w, None, out2, ws)
        sync()
        assert torch.equal(out2, out), f"{label}: without Vhat the sums must be the same bits"
    else:
        with pytest.raises(B.AquaKVError) as e:
            B.aquakv_decode_values_weighted(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], w, None, out, ws)
        assert e.value.status == B.AQUAKV_ENULL
    return out


@pytest.mark.parametrize("dtype,n,layer,batch,S,QH,kind", [
    ("bf16", 16, 1, 2, 512, 24, "softmax"),      # sums taken inside the decode kernel, 2 chunks per sequence
    ("bf16", 64, 1, 1, 768, 64, "any"),          # 8 query heads per kv head
    ("bf16", 256, 1, 3, 256, 8, "any"),          # one query head per kv head
    ("bf16", 16, 1, 2, 150, 32, "softmax"),      # ragged sequences: values decoded to memory first
    ("bf16", 16, 0, 2, 512, 16, "softmax"),      # first layer (no predictor)
    ("fp32", 16, 1, 2, 300, 16, "any"),
    ("fp32", 64, 0, 1, 33, 8, "softmax"),
])
def test_weighted_values(B, dtype, n, layer, batch, S, QH, kind):
    print(f"case weighted dtype={dtype} n={n} layer={layer} batch={batch} S={S} QH={QH} weights={kind}", flush=True)
    H = 8
    cfg = synth.Config("wv", layers=2, kv_heads=H, head_dim=128, tokens=batch * S, dtype=dtype, n_codewords=n)
    Ks, Vs, lo_l, lg_l = P.build_stack(cfg, bias=(n == 64))
    g = P.run_gpu_layers(B, cfg, lg_l, Ks, Vs)[layer]
    w = weights_for(batch, QH, S, 5000 + S + QH, kind)
    fused = dtype == "bf16" and layer == 1 and S % 256 == 0
    check_weighted(B, lo_l[layer], lg_l[layer], g, batch, S, QH, w, fused, "weighted")


@pytest.mark.parametrize("dtype,n,layer,batch,S,QH,spread", [
    ("bf16", 16, 1, 2, 512, 24, 3.0),        # sums and soft-max pieces inside the decode kernel, 2 chunks per sequence
    ("bf16", 64, 1, 1, 1024, 64, 12.0),      # 8 query heads per kv head, peaked rows
    ("bf16", 16, 1, 1, 256, 8, 0.0),         # one chunk, all scores equal: the mean of the values
    ("bf16", 16, 1, 2, 333, 32, 5.0),        # ragged: values decoded to memory first
    ("bf16", 16, 0, 1, 512, 16, 3.0),        # first layer
    ("fp32", 16, 1, 2, 300, 16, 8.0),
])
def test_attend_values(B, dtype, n, layer, batch, S, QH, spread):
    """aquakv_decode_values_attend: soft-max of the scores taken per 256 tokens and merged, against the oracle's
    soft-max rows and weighted sum."""
    print(f"case attend dtype={dtype} n={n} layer={layer} batch={batch} S={S} QH={QH} spread={spread}", flush=True)
    H = 8
    cfg = synth.Config("av", layers=2, kv_heads=H, head_dim=128, tokens=batch * S, dtype=dtype, n_codewords=n)
    Ks, Vs, lo_l, lg_l = P.build_stack(cfg)
    g = P.run_gpu_layers(B, cfg, lg_l, Ks, Vs)[layer]
    lo, lg = lo_l[layer], lg_l[layer]
    gen = torch.Generator().manual_seed(7000 + S + QH)
    # rows with different offsets (the shift must not matter) and a chunk-to-chunk drift so that chunk maxima differ
    s = torch.randn(batch, QH, S, generator=gen) * spread + torch.randn(batch, QH, 1, generator=gen) * 20.0 \
        + torch.linspace(0, spread, S)[None, None, :]
    s = s.float().cuda()
    T = batch * S
    out = torch.full((batch, QH, 128), float("nan"), dtype=torch.float32, device="cuda")
    stats = torch.full((batch, QH, 2), float("nan"), dtype=torch.float32, device="cuda")
    Vout = lg.alloc_kv(T)
    ws = lg.alloc_weighted_workspace(batch, S, QH)
    B.aquakv_decode_values_attend(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], s, Vout, out, stats, ws)
    sync()
    assert torch.equal(P.bits(Vout), P.bits(g["Vhat"]))
    p = O.softmax_rows(U.np64(s))
    vp = None if g["Vp"] is None else U.np64(g["Vp"])
    want, _ = O.attn_values(lo, batch, S, p, g["v_codes"].cpu().numpy(), g["v_scales"].cpu().numpy().view(np.float16), vp,
                            U.np64(g["Khat"]))
    Vh = U.np64(g["Vhat"]).reshape(batch, S, H, 128)
    rep = QH // H
    mag = np.stack([np.einsum("bt,btd->bd", p[:, qh], np.abs(Vh[:, :, qh // rep])) for qh in range(QH)], 1)
    own = np.stack([np.einsum("bt,btd->bd", p[:, qh], Vh[:, :, qh // rep]) for qh in range(QH)], 1)
    got = U.np64(out)
    err, err_own = np.abs(got - want), np.abs(got - own)
    # fp32 exponentials of differences up to a few tens (1e-6 relative each), weights with 16 mantissa bits
    assert np.all(err_own <= 3e-5 * mag + 1e-30), float(np.max(err_own / (mag + 1e-30)))
    # against the oracle the decoded values themselves differ within their storage tolerance, rtol (|v| + rms of the
    # group), and the sum inherits that bound weight by weight
    bound = U.RTOL[dtype] * (mag + np.stack([np.einsum("bt,bt->b", p[:, qh], group_rms(Vh)[:, :, qh // rep]) for qh in range(QH)], 1)[..., None])
    assert np.all(err <= bound + 1e-30), float(np.max(err / (bound + 1e-30)))
    M = U.np64(s).max(axis=-1)
    L = np.exp(U.np64(s) - M[..., None]).sum(axis=-1)
    st = U.np64(stats)
    assert np.array_equal(st[..., 0], M)
    assert np.all(np.abs(st[..., 1] - L) <= 2e-5 * L), float(np.max(np.abs(st[..., 1] - L) / L))
    print(f"   worst error / sum p|v| = {float(np.max(err / (mag + 1e-30))):.3g} against the oracle, "
          f"{float(np.max(err_own / (mag + 1e-30))):.3g} against the sum over the decoded values", flush=True)
    if spread == 0.0:
        assert np.all(np.abs(got - np.stack([Vh[:, :, qh // rep].mean(axis=1) for qh in range(QH)], 1)) <= 3e-5 * mag + 1e-30)
    # the two-call form gives the same result up to the summation
    pr = torch.empty_like(s)
    B.aquakv_softmax(batch * QH, S, s, pr)
    out2 = torch.empty_like(out)
    B.aquakv_decode_values_weighted(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], pr, Vout, out2, ws)
    sync()
    assert np.all(np.abs(U.np64(out2) - got) <= 4e-5 * mag + 1e-30)
    fused = dtype == "bf16" and layer == 1 and S % 256 == 0
    if fused:
        out3 = torch.full_like(out, float("nan"))
        B.aquakv_decode_values_attend(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], s, None, out3, None, ws)
        sync()
        assert torch.equal(out3, out)


def test_attend_every_group_size_of_query_heads(B):
    """1 to 8 query heads per kv head in the decode kernel's epilogue (the head slots of its small matrix product)."""
    H, batch, S = 8, 2, 512
    cfg = synth.Config("gq", layers=2, kv_heads=H, head_dim=128, tokens=batch * S, dtype="bf16", n_codewords=16)
    Ks, Vs, lo_l, lg_l = P.build_stack(cfg)
    g = P.run_gpu_layers(B, cfg, lg_l, Ks, Vs)[1]
    lg = lg_l[1]
    Vh = U.np64(g["Vhat"]).reshape(batch, S, H, 128)
    for rep in range(1, 9):
        QH = H * rep
        print(f"case attend rep={rep}", flush=True)
        gen = torch.Generator().manual_seed(300 + rep)
        s = (torch.randn(batch, QH, S, generator=gen) * 5.0).float().cuda()
        out = torch.full((batch, QH, 128), float("nan"), dtype=torch.float32, device="cuda")
        out_w = torch.full_like(out, float("nan"))
        ws = lg.alloc_weighted_workspace(batch, S, QH)
        B.aquakv_decode_values_attend(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], s, None, out, None, ws)
        w = torch.softmax(s, dim=-1)
        B.aquakv_decode_values_weighted(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], w, None, out_w, ws)
        sync()
        p = O.softmax_rows(U.np64(s))
        own = np.stack([np.einsum("bt,btd->bd", p[:, qh], Vh[:, :, qh // rep]) for qh in range(QH)], 1)
        mag = np.stack([np.einsum("bt,btd->bd", p[:, qh], np.abs(Vh[:, :, qh // rep])) for qh in range(QH)], 1)
        for got in (out, out_w):
            err = np.abs(U.np64(got) - own)
            assert np.all(err <= 3e-5 * mag), (rep, float(np.max(err / mag)))


@pytest.mark.parametrize("bits,rht_group", [(2, None), (4, None), (None, 1024)])
def test_weighted_values_other_quantizers(B, bits, rht_group):
    print(f"case weighted rtn_bits={bits} rht_group={rht_group}", flush=True)
    H, batch, S, QH = 8, 2, 256, 24
    T = batch * S
    D = H * 128
    wk, wv = U.random_weights(D, D, 11, 0.7), U.random_weights(D, 2 * D, 12, 0.7)
    lo0, lg0 = U.make_layers(H, "bf16", 16, layer_idx=0, rtn_bits=bits, rht_group=rht_group)
    lo1, lg1 = U.make_layers(H, "bf16", 16, layer_idx=1, w_k=wk, w_v=wv, rtn_bits=bits, rht_group=rht_group)
    K0, V0, K1, V1 = (P.storage_randn((T, H, 128), "bf16", 60 + i) for i in range(4))
    cfg = synth.Config("wq", layers=2, kv_heads=H, head_dim=128, tokens=T, dtype="bf16", n_codewords=16)
    g = P.run_gpu_layers(B, cfg, [lg0, lg1], [K0, K1], [V0, V1])[1]
    w = weights_for(batch, QH, S, 91, "softmax")
    check_weighted(B, lo1, lg1, g, batch, S, QH, w, fused_expected=True, label="weighted")   # groups of 1024 decode fused too


def test_attention_over_the_compressed_cache_end_to_end(B):
    """scores -> soft-max -> weighted values, every step in the library, against the oracle's attention."""
    print("case attention end to end", flush=True)
    H, QH, batch, S = 8, 32, 2, 512
    cfg = synth.Config("att", layers=2, kv_heads=H, head_dim=128, tokens=batch * S, dtype="bf16", n_codewords=16)
    Ks, Vs, lo_l, lg_l = P.build_stack(cfg)
    g = P.run_gpu_layers(B, cfg, lg_l, Ks, Vs)[1]
    lo, lg = lo_l[1], lg_l[1]
    q = synth.random_queries(batch, QH, 128, seed=78, dtype="bf16", device="cuda")
    scale = 128 ** -0.5
    scores = torch.empty(batch, QH, S, dtype=torch.float32, device="cuda")
    Kout = lg.alloc_kv(cfg.tokens)
    B.aquakv_decode_attn_scores(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, scale, scores, Kout,
                                lg.alloc_workspace(cfg.tokens))
    B.aquakv_softmax(batch * QH, S, scores, scores)
    out = torch.empty(batch, QH, 128, dtype=torch.float32, device="cuda")
    Vout = lg.alloc_kv(cfg.tokens)
    B.aquakv_decode_values_weighted(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], Kout, scores, Vout, out,
                                    lg.alloc_weighted_workspace(batch, S, QH))
    sync()
    cpu = lambda t: t.cpu().numpy()
    s_want = O.attn_scores(lo, batch, S, U.np64(q), cpu(g["k_codes"]), cpu(g["k_scales"]).view(np.float16), U.np64(g["Kp"]), scale)
    p_want = O.softmax_rows(s_want)
    want, _ = O.attn_values(lo, batch, S, p_want, cpu(g["v_codes"]), cpu(g["v_scales"]).view(np.float16), U.np64(g["Vp"]),
                            U.np64(Kout))
    # the output is an average of values: bound relative to the rms of the decoded values
    rms = float(np.sqrt(np.mean(U.np64(Vout) ** 2)))
    err = np.abs(U.np64(out) - want)
    assert err.max() <= U.RTOL["bf16"] * rms, (err.max(), rms)
    print(f"   worst |error| / rms(V) = {err.max() / rms:.3g}", flush=True)
    # the three-launch form: scores with the keys, then the values with the soft-max inside
    B.aquakv_decode_attn_scores(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, scale, scores, Kout,
                                lg.alloc_workspace(cfg.tokens))
    out2 = torch.empty_like(out)
    B.aquakv_decode_values_attend(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], Kout, scores, Vout, out2, None,
                                  lg.alloc_weighted_workspace(batch, S, QH))
    sync()
    err2 = np.abs(U.np64(out2) - want)
    assert err2.max() <= U.RTOL["bf16"] * rms, (err2.max(), rms)
    print(f"   soft-max inside: worst |error| / rms(V) = {err2.max() / rms:.3g}", flush=True)


@pytest.mark.parametrize("S,QH", [(8192, 24), (32768, 32)])
def test_weighted_values_at_the_bench_shapes(B, S, QH):
    """The launch configurations the benchmark times (8192 tokens with 24 query heads, 32768 with 32; 8 kv heads,
    n = 16): both forms against the fp64 sums over the values the same call wrote, whose rows other tests check
    against the oracle."""
    print(f"case weighted at {S} tokens, {QH} query heads", flush=True)
    H, batch = 8, 1
    rep = QH // H
    cfg = synth.Config("wb", layers=2, kv_heads=H, head_dim=128, tokens=S, dtype="bf16", n_codewords=16)
    Ks, Vs, lo_l, lg_l = P.build_stack(cfg)
    g = P.run_gpu_layers(B, cfg, lg_l, Ks, Vs)[1]
    lg = lg_l[1]
    gen = torch.Generator().manual_seed(17)
    scores = (torch.randn(batch, QH, S, generator=gen) * 4.0 + torch.linspace(-3, 3, S)[None, None, :]).float().cuda()
    w = torch.softmax(scores, dim=-1)
    out = torch.empty(batch, QH, 128, dtype=torch.float32, device="cuda")
    out2 = torch.empty_like(out)
    stats = torch.empty(batch, QH, 2, dtype=torch.float32, device="cuda")
    Vout = lg.alloc_kv(S)
    ws = lg.alloc_weighted_workspace(batch, S, QH)
    B.aquakv_decode_values_weighted(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], w, Vout, out, ws)
    sync()
    assert torch.equal(P.bits(Vout), P.bits(g["Vhat"]))
    Vout.zero_()
    B.aquakv_decode_values_attend(lg, batch, S, QH, g["v_codes"], g["v_scales"], g["Vp"], g["Khat"], scores, Vout, out2, stats, ws)
    sync()
    assert torch.equal(P.bits(Vout), P.bits(g["Vhat"]))
    Vh = U.np64(Vout).reshape(S, H, 128)
    for got, wd, tol in ((out, U.np64(w)[0], 2e-5), (out2, O.softmax_rows(U.np64(scores))[0], 3e-5)):
        own = np.stack([wd[qh] @ Vh[:, qh // rep] for qh in range(QH)])
        mag = np.stack([np.abs(wd[qh]) @ np.abs(Vh[:, qh // rep]) for qh in range(QH)])
        err = np.abs(U.np64(got)[0] - own)
        assert np.all(err <= tol * mag), float(np.max(err / mag))
        print(f"   worst error / sum|w||v| = {float(np.max(err / mag)):.3g}", flush=True)
    sd = U.np64(scores)[0]
    assert np.array_equal(U.np64(stats)[0, :, 0], sd.max(axis=1))
    Lw = np.exp(sd - sd.max(axis=1, keepdims=True)).sum(axis=1)
    assert np.all(np.abs(U.np64(stats)[0, :, 1] - Lw) <= 2e-5 * Lw)
