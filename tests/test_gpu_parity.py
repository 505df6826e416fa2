"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element
by element on the same seeded inputs.  Codes and scales must be bit-exact except
for counted ties; reconstructions within 1e-5 (fp32) / 2e-2 (bf16) relative."""
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


def storage_randn(shape, dtype, seed, scale=1.0, device="cuda"):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(*shape, generator=g) * scale).to(synth.torch_dtype(dtype)).to(device)


def sync():
    torch.cuda.synchronize()


# ------------------------------------------------------------------ predictor
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("T,H", [(1, 2), (300, 2), (515, 8)])
def test_predict_matches_oracle_and_is_row_count_invariant(B, dtype, T, H):
    print(f"case predict dtype={dtype} T={T} H={H}", flush=True)
    D = H * 128
    wk = U.random_weights(D, D, 1)
    wv = U.random_weights(D, 2 * D, 2)
    bk = torch.randn(D, generator=torch.Generator().manual_seed(3))
    lo, lg = U.make_layers(H, dtype, 16, w_k=wk, w_v=wv, b_k=bk)
    x0 = storage_randn((T, D), dtype, 4)
    x1 = storage_randn((T, D), dtype, 5)
    P = torch.empty(T, D, dtype=torch.float32, device="cuda")
    for which, a0, a1, W, b in ((B.AQUAKV_KEY, x0, None, lo.w_k, lo.b_k), (B.AQUAKV_VALUE, x0, x1, lo.w_v, lo.b_v)):
        B.aquakv_predict(lg, which, T, a0, a1, P)
        sync()
        xin = U.np64(a0) if a1 is None else np.concatenate([U.np64(a0), U.np64(a1)], axis=1)
        want = O.predict(xin, W, b)
        mag = np.abs(xin) @ np.abs(W).T + (0 if b is None else np.abs(b))
        err = np.abs(U.np64(P) - want)
        assert np.all(err <= 4e-6 * mag + 1e-30), float(np.max(err / (mag + 1e-30)))
        # the same rows alone (a different launch shape) give the same bits
        rows = [0, T // 2, T - 1]
        for r in rows:
            P1 = torch.empty(1, D, dtype=torch.float32, device="cuda")
            B.aquakv_predict(lg, which, 1, a0[r:r + 1].contiguous(), None if a1 is None else a1[r:r + 1].contiguous(), P1)
            sync()
            assert torch.equal(P1[0], P[r])


# ------------------------------------------------------------------ quantizer stages
@pytest.mark.parametrize("dtype,n,T,H", [("fp32", 16, 256, 2), ("bf16", 16, 300, 8), ("bf16", 64, 257, 8),
                                        ("fp32", 64, 33, 2), ("bf16", 256, 65, 4), ("fp32", 16, 1, 1)])
@pytest.mark.parametrize("with_p,table", [(False, True), (True, True), (True, False)])
def test_quantize_codes_scales_and_reconstruction(B, dtype, n, T, H, with_p, table):
    print(f"case quantize dtype={dtype} n={n} T={T} H={H} with_p={with_p} table={table}", flush=True)
    lo, lg = U.make_layers(H, dtype, n, table=table)
    D = H * 128
    ch = synth.channel_scales(D, 0, 0).float()
    X = (storage_randn((T, D), "fp32", 10, device="cpu") * ch).to(synth.torch_dtype(dtype)).cuda().reshape(T, H, 128)
    P = (storage_randn((T, D), "fp32", 11) * 0.8).reshape(T, H, 128).contiguous() if with_p else None
    for which, signs in ((B.AQUAKV_KEY, lo.signs_k), (B.AQUAKV_VALUE, lo.signs_v)):
        codes, scales = lg.alloc_codes(T)
        Xhat = lg.alloc_kv(T)
        B.aquakv_quantize(lg, which, T, X, P, codes, scales, Xhat)
        sync()
        p64 = np.zeros((T, H, 128)) if P is None else U.np64(P)
        rep = U.compare_quantizer_outputs(U.np64(X) - p64, signs, lo.codebook, codes.cpu().numpy(),
                                          scales.cpu().numpy(), n)
        print("  ", rep, flush=True)
        assert rep.other == 0, str(rep)
        assert rep.code_mismatch <= max(2, rep.subvectors // 20000) and rep.scale_mismatch <= max(1, rep.groups // 500)
        # the reconstruction is the oracle's decode of the GPU's own codes
        g_idx = O.unpack_codes(codes.cpu().numpy(), n)
        g_s16 = scales.cpu().numpy().view(np.float16)
        want = O.round_storage(O.dequantize(g_idx, g_s16, signs, lo.codebook) + p64, dtype)
        U.assert_close_storage(Xhat, want, dtype, "Xhat")
        # and bit-identical to what the dequantize entry point gives
        X2 = lg.alloc_kv(T)
        B.aquakv_dequantize(lg, which, T, codes, scales, P, X2)
        sync()
        assert torch.equal(X2.view(torch.int16 if dtype == "bf16" else torch.int32),
                           Xhat.view(torch.int16 if dtype == "bf16" else torch.int32))


@pytest.mark.parametrize("dtype,n", [("fp32", 16), ("bf16", 64), ("bf16", 256)])
def test_dequantize_random_codes(B, dtype, n):
    print(f"case dequantize dtype={dtype} n={n}", flush=True)
    T, H = 131, 8
    lo, lg = U.make_layers(H, dtype, n)
    rng = np.random.Generator(np.random.PCG64(12))
    idx = rng.integers(0, n, size=(T, H, 64))
    s16 = (np.abs(rng.standard_normal((T, H))) * 10 ** rng.uniform(-3, 2, (T, H))).astype(np.float16)
    s16[0, 0] = 0
    codes = torch.from_numpy(O.pack_codes(idx, n)).cuda()
    scales = torch.from_numpy(s16.view(np.int16)).cuda()
    P = (storage_randn((T, H * 128), "fp32", 13) * 3).reshape(T, H, 128).contiguous()
    Xhat = lg.alloc_kv(T)
    B.aquakv_dequantize(lg, B.AQUAKV_VALUE, T, codes, scales, P, Xhat)
    sync()
    want = O.round_storage(O.dequantize(idx, s16, lo.signs_v, lo.codebook) + U.np64(P), dtype)
    U.assert_close_storage(Xhat, want, dtype, "dequantize")


@pytest.mark.parametrize("n", [16, 64, 256])
def test_search_table_gives_the_codes_of_the_full_search(B, n):
    """Same kernel with and without the table, on inputs that also reach the border cells."""
    print(f"case table vs full search n={n}", flush=True)
    T, H = 2048, 8
    _, lg_t = U.make_layers(H, "fp32", n, table=True)
    _, lg_f = U.make_layers(H, "fp32", n, table=False)
    g = torch.Generator().manual_seed(31)
    X = torch.randn(T, H, 128, generator=g)
    X[: T // 2] *= torch.exp(2.5 * torch.randn(T // 2, H, 128, generator=g))     # heavy tails -> |y| up to ~11
    X[T // 2: T // 2 + 64, :, 1:] = 0                                             # a single spike per group
    X = X.cuda()
    outs = []
    for lg in (lg_t, lg_f):
        codes, scales = lg.alloc_codes(T)
        B.aquakv_quantize(lg, B.AQUAKV_KEY, T, X, None, codes, scales, None)
        sync()
        outs.append((codes, scales))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    # Cells with more candidates than the kernels score per cell name an overflow list (up to 8 candidates) or, beyond
    # that, the full search.  Layout of the table words: 64 x 64 cell entries, then 128 lists of two words.
    from paper_2501_19392_amd import binding
    shift = 4 if n == 16 else 0
    top = (n - 1) << shift
    crowded = 0xFF000000 if n == 256 else (top + 1) << 24               # entries >= this are crowded
    full_mark = 0xFF000000 | (top << 16) | (top << 8) | top
    def split(tab):
        w = tab.cpu().numpy().view(np.uint32)
        assert w.size == 64 * 64 + 2 * 128
        cells = w[:4096]
        return cells, (cells >= crowded) & (cells != full_mark), cells == full_mark, w[4096:]
    cells, listed, full, lists = split(lg_t.search_table)
    print(f"   regular grid: {int(listed.sum())} cells with an overflow list, {int(full.sum())} left to the full search", flush=True)
    assert full.sum() == 0 and listed.sum() >= {16: 1, 64: 3, 256: 8}[n]
    for e in cells[listed]:                      # a list is ascending with its last candidate repeated
        k = int(e & 0xff) >> shift
        c = np.concatenate([lists[2 * k: 2 * k + 2].view(np.uint8)]).astype(int)
        assert np.all(np.diff(c) >= 0) and np.all(c % (1 << shift) == 0) and c.max() <= top
        assert len(set(c.tolist())) >= 2 or (n == 256 and k == 0 and c[0] == 255)      # (the list shared by the cells of point 255 alone)
    # rows built so that their normalised rotated pairs fall into the centres of the cells with overflow lists (random
    # inputs reach those of the 16- and 64-point grids about once in 1e8 pairs): x = s * H y / sqrt(128) with rms(y) = 1
    from scipy.linalg import hadamard
    Hm = hadamard(128).astype(np.float64)
    cyx = np.argwhere(listed.reshape(64, 64))
    R = 3.25 if n == 256 else 4.0                                                   # the table's range for this grid
    centres = np.stack([-R + (cyx[:, 1] + 0.5) * (R / 32), -R + (cyx[:, 0] + 0.5) * (R / 32)], 1)     # (y0, y1) per cell
    rng = np.random.Generator(np.random.PCG64(5))
    rows = np.zeros((256, H, 128))
    hit = 0
    for r in range(256):
        for h in range(H):
            y = np.zeros((64, 2))
            budget, m = 128.0, 0
            for c in centres[rng.permutation(len(centres))]:
                if m < 40 and budget - float(c @ c) > 0.02 * (63 - m):
                    y[m] = c; budget -= float(c @ c); m += 1
            y[m:] = np.sqrt(budget / (2 * (64 - m))) * rng.choice([-1.0, 1.0], size=(64 - m, 2))
            hit += m
            sg = np.where(lg_t.signs_k.cpu().numpy().reshape(H, 128)[h] < 0, -1.0, 1.0)
            rows[r, h] = sg * (Hm @ y.reshape(128)) / np.sqrt(128.0)
    assert hit >= 256 * H            # at least one targeted pair per group on average
    Xc = torch.from_numpy(rows).float().cuda()
    got = []
    for lg in (lg_t, lg_f):
        codes, scales = lg.alloc_codes(256)
        B.aquakv_quantize(lg, B.AQUAKV_KEY, 256, Xc, None, codes, scales, None)
        sync()
        got.append((codes, scales))
    assert torch.equal(got[0][0], got[1][0]) and torch.equal(got[0][1], got[1][1])
    print(f"   {hit} pairs aimed at cells with overflow lists: codes equal those of the full search", flush=True)
    # a crowded grid (many points inside one cell) runs out of lists, takes the full-search fallback and still agrees
    C = torch.from_numpy(synth.lloyd_codebook(n)).clone()
    C[: n // 2] = C[: n // 2] * 0.01
    Cd = C.cuda()
    tab = binding.build_search_table(Cd)
    _, listed_c, full_c, _ = split(tab)
    assert full_c.sum() > 0 and (n == 16 or listed_c.sum() > 0)
    res = []
    for t in (tab, None):
        lg = binding.Layer(H, 128, Cd, lg_t.signs_k, lg_t.signs_v, torch.float32, search_table=t)
        codes, scales = lg.alloc_codes(T)
        B.aquakv_quantize(lg, B.AQUAKV_KEY, T, X, None, codes, scales, None)
        sync()
        res.append(codes)
    assert torch.equal(res[0], res[1])


@pytest.mark.parametrize("n", [16, 64, 256])
def test_search_table_lists_the_candidates_of_every_cell(B, n):
    """The table against its definition, cell by cell, in numpy: grid point j belongs to a cell unless one other point
    i is closer by more than eps at all four corners of the slightly enlarged cell (the difference of two squared
    distances is linear, so the corners decide).  A cell entry, or the overflow list it names, must hold exactly
    that set, ascending; all cells for the two small grids, the crowded ones and a seeded sample for the 256-point grid."""
    print(f"case table contents n={n}", flush=True)
    from paper_2501_19392_amd import binding
    C32 = np.ascontiguousarray(synth.lloyd_codebook(n), dtype=np.float32).reshape(n, 2)
    C = C32.astype(np.float64)                                       # the values the builder reads
    tab = binding.build_search_table(torch.from_numpy(C32).cuda())
    sync()
    w = tab.cpu().numpy().view(np.uint32)
    cells, lists = w[:4096], w[4096:]
    shift = 4 if n == 16 else 0
    top = (n - 1) << shift
    crowded = 0xFF000000 if n == 256 else (top + 1) << 24
    full_mark = 0xFF000000 | (top << 16) | (top << 8) | top
    R = 3.25 if n == 256 else 4.0
    h, far, delta, eps = 2 * R / 64, 1e30, 1e-4, 1e-3
    A, Bv = C[:, 0][:, None], C[:, 1][:, None]
    gx, gy = -2 * (A - A.T), -2 * (Bv - Bv.T)
    c0 = (A * A + Bv * Bv) - (A * A + Bv * Bv).T                      # [j, i]: d_j - d_i = gx x + gy y + c0
    if n == 256:
        rng = np.random.Generator(np.random.PCG64(11))
        todo = sorted(set(np.nonzero(cells >= crowded)[0].tolist()[:150] + rng.choice(4096, 250, replace=False).tolist()
                          + [0, 63, 4032, 4095, 2080]))
    else:
        todo = range(4096)
    for cell in todo:
        cx, cy = cell % 64, cell // 64
        x0 = -far if cx == 0 else -R + cx * h
        x1 = far if cx == 63 else -R + (cx + 1) * h
        y0 = -far if cy == 0 else -R + cy * h
        y1 = far if cy == 63 else -R + (cy + 1) * h
        xs = np.array([x0 - delta, x1 + delta, x0 - delta, x1 + delta])
        ys = np.array([y0 - delta, y0 - delta, y1 + delta, y1 + delta])
        mn = np.min(gx[:, :, None] * xs + gy[:, :, None] * ys + c0[:, :, None], axis=2)
        np.fill_diagonal(mn, -1.0)
        want = np.nonzero(~(mn > eps).any(axis=1))[0].tolist()
        e = int(cells[cell])
        if e >= crowded:
            assert e != full_mark, cell
            k = (e & 0xff) >> shift
            got = lists[2 * k: 2 * k + 2].view(np.uint8).astype(int)
            assert len(want) > (3 if n == 16 else 4) or (n == 256 and want[-1] == 255), (cell, want)
        else:
            got = np.array([e & 0xff, (e >> 8) & 0xff, (e >> 16) & 0xff, e >> 24])
        got = (got >> shift).tolist()
        assert np.all(np.diff(got) >= 0) and sorted(set(got)) == want, (cell, got, want)
        assert got[len(want) - 1:] == [want[-1]] * (len(got) - len(want) + 1), (cell, got)     # the last one repeated
    print(f"   {len(todo)} cells: candidate sets as defined", flush=True)


def test_quantize_edge_cases(B):
    """Zero residual, huge values (scale clamps at the fp16 maximum), tiny values (subnormal
    fp16 scales), in-place reconstruction, and a row count that leaves most of a block idle."""
    print("case quantize edge cases", flush=True)
    H, n, T = 2, 16, 5
    lo, lg = U.make_layers(H, "fp32", n)
    X = storage_randn((T, H, 128), "fp32", 20)
    X[1] *= 3e6          # sigma above 65504 -> clamped
    X[2] *= 1e-6         # sigma in the fp16 subnormal range
    X[3] = 0             # zero residual
    P = torch.zeros_like(X)
    P[4] = X[4]          # residual exactly zero with a non-zero prediction
    codes, scales = lg.alloc_codes(T)
    Xhat = X.clone()
    B.aquakv_quantize(lg, B.AQUAKV_KEY, T, Xhat, P, codes, scales, Xhat)      # in place
    sync()
    s16 = scales.cpu().numpy().view(np.float16)
    assert np.all(s16[1] == np.float16(65504)) and np.all(s16[3] == 0) and np.all(s16[4] == 0)
    assert np.all(s16[2] > 0) and np.all(s16[2] < 6.2e-5)
    rep = U.compare_quantizer_outputs(U.np64(X) - U.np64(P), lo.signs_k, lo.codebook, codes.cpu().numpy(),
                                      scales.cpu().numpy(), n)
    print("  ", rep, flush=True)
    assert rep.other == 0 and rep.code_mismatch == 0 and rep.scale_mismatch == 0, str(rep)
    assert torch.equal(Xhat[3], torch.zeros_like(Xhat[3])) and torch.equal(Xhat[4], X[4])
    g_idx = O.unpack_codes(codes.cpu().numpy(), n)
    want = O.round_storage(O.dequantize(g_idx, s16, lo.signs_k, lo.codebook) + U.np64(P), "fp32")
    U.assert_close_storage(Xhat, want, "fp32", "edge Xhat")
    # tokens = 0: nothing is touched
    B.aquakv_quantize(lg, B.AQUAKV_KEY, 0, X, None, codes, scales, None)
    sync()


# ------------------------------------------------------------------ whole layers
def run_gpu_layers(B, cfg, layers_g, Ks, Vs, want_hat=True):
    """encode every layer in order on the GPU, feeding reconstructions forward."""
    T = Ks[0].shape[0]
    out = []
    Kp = Vp = None
    for l, lg in enumerate(layers_g):
        kc, ks = lg.alloc_codes(T)
        vc, vs = lg.alloc_codes(T)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        ws = lg.alloc_workspace(T)
        B.aquakv_encode_layer(lg, T, Ks[l], Vs[l], Kp, Vp, kc, ks, vc, vs, Kh, Vh, ws)
        sync()
        out.append(dict(k_codes=kc, k_scales=ks, v_codes=vc, v_scales=vs, Khat=Kh, Vhat=Vh, Kp=Kp, Vp=Vp))
        Kp, Vp = Kh, Vh
    return out


def build_stack(cfg, device="cuda", predictors="analytic", bias=False, rht_group=None):
    st = synth.KVStream(cfg, device="cpu", work=torch.float64)
    Ks, Vs, lo_l, lg_l = [], [], [], []
    for l in range(cfg.layers):
        K, V = st.next()
        Ks.append(K.to(device))
        Vs.append(V.to(device))
        if l == 0:
            lo, lg = U.make_layers(cfg.kv_heads, cfg.dtype, cfg.n_codewords, layer_idx=l, rht_group=rht_group)
        else:
            if predictors == "analytic":
                wk, wv = synth.analytic_predictors(st, l)
            else:
                wk, wv = U.random_weights(cfg.d, cfg.d, 100 + l, 0.7), U.random_weights(cfg.d, 2 * cfg.d, 200 + l, 0.7)
            gb = torch.Generator().manual_seed(300 + l)
            bk = torch.randn(cfg.d, generator=gb) * 0.3 if bias else None
            bv = torch.randn(cfg.d, generator=gb) * 0.3 if bias else None
            lo, lg = U.make_layers(cfg.kv_heads, cfg.dtype, cfg.n_codewords, layer_idx=l, w_k=wk, w_v=wv, b_k=bk, b_v=bv,
                                   rht_group=rht_group)
        lo_l.append(lo)
        lg_l.append(lg)
    return Ks, Vs, lo_l, lg_l


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def check_layer_against_oracle(B, lo, lg, K, V, g, rows=None):
    """One layer, teacher-forced at every stage boundary with the GPU's own tensors:
    each stage of the GPU result must match the oracle given the same inputs."""
    n = lo.n_codewords
    sel = slice(None) if rows is None else rows
    T = K.shape[0]
    D = lo.kv_heads * lo.head_dim
    shape = (-1, lo.groups_per_token, lo.group)           # rotation groups: one per head, or the whole token
    reports = []
    for which, X, codes, scales, hat, signs in (
            ("k", K, g["k_codes"], g["k_scales"], g["Khat"], lo.signs_k),
            ("v", V, g["v_codes"], g["v_scales"], g["Vhat"], lo.signs_v)):
        has = (lo.w_k if which == "k" else lo.w_v) is not None
        if has:
            P = torch.empty(T, D, dtype=torch.float32, device="cuda")
            if which == "k":
                B.aquakv_predict(lg, B.AQUAKV_KEY, T, g["Kp"], None, P)
                xin = U.np64(g["Kp"][sel]).reshape(-1, D)
                want_p = O.predict(xin, lo.w_k, lo.b_k)
                W = lo.w_k
            else:
                B.aquakv_predict(lg, B.AQUAKV_VALUE, T, g["Vp"], g["Khat"], P)
                xin = np.concatenate([U.np64(g["Vp"][sel]).reshape(-1, D), U.np64(g["Khat"][sel]).reshape(-1, D)], 1)
                want_p = O.predict(xin, lo.w_v, lo.b_v)
                W = lo.w_v
            sync()
            p64 = U.np64(P[sel])
            mag = np.abs(xin) @ np.abs(W).T
            assert np.all(np.abs(p64 - want_p) <= 4e-6 * mag + 1e-30)
            p64 = p64.reshape(shape)
        else:
            p64 = np.zeros((U.np64(X[sel]).reshape(shape)).shape)
        x64 = U.np64(X[sel]).reshape(shape)
        c = codes[sel].cpu().numpy().reshape(x64.shape[0], lo.groups_per_token, -1)
        s = scales[sel].cpu().numpy()
        signs = np.asarray(signs).reshape(lo.groups_per_token, lo.group)
        rep = U.compare_quantizer_outputs(x64 - p64, signs, lo.codebook, c, s, n)
        reports.append(rep)
        assert rep.other == 0, f"{which}: {rep}"
        want = O.round_storage(O.dequantize(O.unpack_codes(c, n), s.view(np.float16), signs, lo.codebook) + p64, lo.dtype)
        U.assert_close_storage(hat[sel], want, lo.dtype, which + "hat")
    return reports


def free_run_layers(B, lo_l, lg_l, Ks, Vs, out, rows=None):
    """The oracle's own sweep over the layers (its reconstructions feeding its next predictions, no teacher forcing)
    beside the library's, on the token rows `rows` (tokens are independent): [(layer, "k" | "v", FreeRunReport)]."""
    sel = slice(None) if rows is None else rows
    reports = []
    free_run_layers.last_oracle = []
    Kp = Vp = None
    for l, (lo, lg) in enumerate(zip(lo_l, lg_l)):
        g = out[l]
        T = Ks[l].shape[0]
        D = lo.kv_heads * lo.head_dim
        K64, V64 = U.np64(Ks[l][sel]), U.np64(Vs[l][sel])
        e = O.encode_layer(lo, K64, V64, Kp, Vp)
        free_run_layers.last_oracle.append(e)
        shape = (-1, lo.groups_per_token, lo.group)
        for which, X64, codes, scales, signs in (("k", K64, g["k_codes"], g["k_scales"], lo.signs_k),
                                                 ("v", V64, g["v_codes"], g["v_scales"], lo.signs_v)):
            has = (lo.w_k if which == "k" else lo.w_v) is not None
            if has:
                # the library's own prediction (same main loop as its fused kernels) and the oracle's from its own sweep
                P = torch.empty(T, D, dtype=torch.float32, device="cuda")
                if which == "k":
                    B.aquakv_predict(lg, B.AQUAKV_KEY, T, g["Kp"], None, P)
                else:
                    B.aquakv_predict(lg, B.AQUAKV_VALUE, T, g["Vp"], g["Khat"], P)
                sync()
                p_g = U.np64(P[sel]).reshape(shape)
                p_o = e["P_k" if which == "k" else "P_v"].reshape(shape)
            else:
                p_g = p_o = np.zeros(X64.reshape(shape).shape)
            c = codes[sel].cpu().numpy().reshape(p_g.shape[0], lo.groups_per_token, -1)
            rep = U.classify_free_run(X64.reshape(shape), p_o, p_g, np.asarray(signs).reshape(lo.groups_per_token, lo.group),
                                      lo.codebook, c, scales[sel].cpu().numpy(), lo.n_codewords)
            reports.append((l, which, rep))
        Kp, Vp = e["Khat"], e["Vhat"]
    return reports


@pytest.mark.parametrize("predictors", ["analytic", "random"])
def test_tiny_config_fp32_end_to_end(B, predictors):
    """Config 'Tiny' in full: every stage of every layer against the oracle, then the free-running
    oracle (no teacher forcing), then decode reproduces encode bit for bit."""
    print(f"case tiny e2e predictors={predictors}", flush=True)
    cfg = synth.TINY
    Ks, Vs, lo_l, lg_l = build_stack(cfg, predictors=predictors)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    for l in range(cfg.layers):
        for rep in check_layer_against_oracle(B, lo_l[l], lg_l[l], Ks[l], Vs[l], out[l]):
            print(f"   layer {l}: {rep}", flush=True)
    # free-running oracle over both layers: every disagreement is put down to a cause, none may be left over
    reports = free_run_layers(B, lo_l, lg_l, Ks, Vs, out)
    for l, which, rep in reports:
        print(f"   free-run layer {l} {which}: {rep}", flush=True)
        assert rep.other == 0, f"layer {l} {which}: {rep}"
        # fp32 mode: the inputs of the two quantizers differ by fp32 accumulation (<= 4e-6 sum |x||w| per prediction)
        # and by the fp32 rounding of the reconstructions upstream; in normalised units that stays below 1e-3
        # (256 .. 512 products of about 0.04 |x|, residual rms about 0.4 |x|), and disagreements are rare
        assert rep.max_input_diff <= 1e-3, str(rep)
        assert rep.code_mismatch <= max(2, rep.subvectors // 2000) and rep.scale_mismatch <= max(1, rep.groups // 200), str(rep)
    for l in range(cfg.layers):
        e = free_run_layers.last_oracle[l]
        for name in ("Khat", "Vhat"):
            rel = np.linalg.norm(U.np64(out[l][name]) - e[name]) / np.linalg.norm(e[name])
            assert rel < 2e-3, rel
    # closed loop
    for l in range(cfg.layers):
        g, lg = out[l], lg_l[l]
        Kh, Vh = lg.alloc_kv(cfg.tokens), lg.alloc_kv(cfg.tokens)
        B.aquakv_decode_layer(lg, cfg.tokens, g["k_codes"], g["k_scales"], g["v_codes"], g["v_scales"], g["Kp"], g["Vp"],
                              Kh, Vh, lg.alloc_workspace(cfg.tokens))
        sync()
        assert torch.equal(bits(Kh), bits(g["Khat"])) and torch.equal(bits(Vh), bits(g["Vhat"]))


@pytest.mark.parametrize("n", [16, 64])
def test_bf16_three_layers_ragged(B, n):
    print(f"case bf16 3 layers n={n}", flush=True)
    cfg = synth.Config("mid", layers=3, kv_heads=8, head_dim=128, tokens=389, dtype="bf16", n_codewords=n)
    Ks, Vs, lo_l, lg_l = build_stack(cfg)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    for l in range(cfg.layers):
        for rep in check_layer_against_oracle(B, lo_l[l], lg_l[l], Ks[l], Vs[l], out[l]):
            print(f"   layer {l}: {rep}", flush=True)
        g, lg = out[l], lg_l[l]
        Kh, Vh = lg.alloc_kv(cfg.tokens), lg.alloc_kv(cfg.tokens)
        B.aquakv_decode_layer(lg, cfg.tokens, g["k_codes"], g["k_scales"], g["v_codes"], g["v_scales"], g["Kp"], g["Vp"],
                              Kh, Vh, lg.alloc_workspace(cfg.tokens))
        sync()
        assert torch.equal(bits(Kh), bits(g["Khat"])) and torch.equal(bits(Vh), bits(g["Vhat"]))
        # decoding a sub-range of rows on its own gives the same bits (append path, M-independence)
        r0, r1 = 100, 164
        Kh2, Vh2 = lg.alloc_kv(r1 - r0), lg.alloc_kv(r1 - r0)
        cut = lambda t: None if t is None else t[r0:r1].contiguous()
        B.aquakv_decode_layer(lg, r1 - r0, cut(g["k_codes"]), cut(g["k_scales"]), cut(g["v_codes"]), cut(g["v_scales"]),
                              cut(g["Kp"]), cut(g["Vp"]), Kh2, Vh2, lg.alloc_workspace(r1 - r0))
        sync()
        assert torch.equal(bits(Kh2), bits(g["Khat"][r0:r1])) and torch.equal(bits(Vh2), bits(g["Vhat"][r0:r1]))
    # the quality claim of Sect. 3.1 on the GPU's own output: predictors cut the error several-fold
    K2 = U.np64(Ks[2])
    err_pred = np.sum((U.np64(out[2]["Khat"]) - K2) ** 2) / np.sum(K2 ** 2)
    assert err_pred < (0.06 if n == 16 else 0.02), err_pred


@pytest.mark.parametrize("dtype,H,T", [("bf16", 1, 1), ("bf16", 1, 255), ("bf16", 3, 256), ("bf16", 5, 257), ("bf16", 16, 300),
                                       ("bf16", 6, 513), ("fp32", 3, 130), ("fp32", 16, 65)])
def test_head_counts_and_tile_edges(B, dtype, H, T):
    """Head counts other than 8 (odd ones: the workgroup count is then not a multiple of the 8 XCDs; 16: predictor
    inputs of 2048 / 4096) at token counts around the edges of the 256-row tile: every stage against the oracle,
    decode reproduces encode bit for bit, scores against the decoded keys."""
    print(f"case head counts dtype={dtype} H={H} T={T}", flush=True)
    cfg = synth.Config("shapes", layers=2, kv_heads=H, head_dim=128, tokens=T, dtype=dtype)
    Ks, Vs, lo_l, lg_l = build_stack(cfg, predictors="random", bias=True)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    for l in range(cfg.layers):
        for rep in check_layer_against_oracle(B, lo_l[l], lg_l[l], Ks[l], Vs[l], out[l]):
            print(f"   layer {l}: {rep}", flush=True)
        g, lg = out[l], lg_l[l]
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        ws = lg.alloc_workspace(T)
        B.aquakv_decode_layer(lg, T, g["k_codes"], g["k_scales"], g["v_codes"], g["v_scales"], g["Kp"], g["Vp"], Kh, Vh, ws)
        sync()
        assert torch.equal(bits(Kh), bits(g["Khat"])) and torch.equal(bits(Vh), bits(g["Vhat"]))
        QH = 2 * H
        q = synth.random_queries(1, QH, 128, seed=7, dtype=dtype, device="cuda")
        scores = torch.empty(1, QH, T, dtype=torch.float32, device="cuda")
        B.aquakv_decode_attn_scores(lg, 1, T, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 1.0, scores, None, ws)
        sync()
        k64 = np.repeat(U.np64(g["Khat"]), 2, axis=1)
        want = np.einsum("qd,tqd->qt", U.np64(q)[0], k64)
        mag = np.einsum("qd,tqd->qt", np.abs(U.np64(q)[0]), np.abs(k64))
        assert np.all(np.abs(U.np64(scores)[0] - want) <= U.RTOL[dtype] * mag + 1e-30)


def test_encode_without_optional_outputs_matches(B):
    """Khat / Vhat may be NULL: codes and scales must not change."""
    print("case optional outputs", flush=True)
    cfg = synth.Config("opt", layers=2, kv_heads=2, head_dim=128, tokens=77, dtype="bf16")
    Ks, Vs, lo_l, lg_l = build_stack(cfg)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    g, lg, T = out[1], lg_l[1], cfg.tokens
    kc, ks = lg.alloc_codes(T)
    vc, vs = lg.alloc_codes(T)
    B.aquakv_encode_layer(lg, T, Ks[1], Vs[1], g["Kp"], g["Vp"], kc, ks, vc, vs, None, None, lg.alloc_workspace(T))
    sync()
    for a, b in ((kc, g["k_codes"]), (ks, g["k_scales"]), (vc, g["v_codes"]), (vs, g["v_scales"])):
        assert torch.equal(a, b)
    # keys only decode
    Kh = lg.alloc_kv(T)
    B.aquakv_decode_layer(lg, T, kc, ks, None, None, g["Kp"], None, Kh, None, lg.alloc_workspace(T))
    sync()
    assert torch.equal(bits(Kh), bits(g["Khat"]))


def test_encode_layer_in_place(B):
    """Khat may alias K and Vhat may alias V (the reconstruction overwrites the raw tensor): same codes, same
    reconstructions as out of place, in the fused bf16 path (predicted layer) and the stand-alone path (layer 0)."""
    print("case encode in place", flush=True)
    cfg = synth.Config("inplace", layers=2, kv_heads=8, head_dim=128, tokens=517, dtype="bf16", n_codewords=16)
    Ks, Vs, lo_l, lg_l = build_stack(cfg)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    T = cfg.tokens
    for l, lg in enumerate(lg_l):
        g = out[l]
        K2, V2 = Ks[l].clone(), Vs[l].clone()
        kc, ks = lg.alloc_codes(T)
        vc, vs = lg.alloc_codes(T)
        B.aquakv_encode_layer(lg, T, K2, V2, g["Kp"], g["Vp"], kc, ks, vc, vs, K2, V2, lg.alloc_workspace(T))
        sync()
        assert torch.equal(kc, g["k_codes"]) and torch.equal(ks, g["k_scales"])
        assert torch.equal(vc, g["v_codes"]) and torch.equal(vs, g["v_scales"])
        assert torch.equal(bits(K2), bits(g["Khat"])) and torch.equal(bits(V2), bits(g["Vhat"]))


@pytest.mark.parametrize("dtype,rht_group", [("bf16", None), ("fp32", None), ("bf16", 1024)])
def test_key_and_value_halves_on_two_streams(B, dtype, rht_group):
    """aquakv_encode_keys / aquakv_encode_values / aquakv_decode_values (+ keys-only aquakv_decode_layer): the key
    chain on one stream, the value chain on another with an event per layer, give the same bytes as the layer calls."""
    print(f"case halves dtype={dtype} rht_group={rht_group}", flush=True)
    H = 8 if dtype == "bf16" else 2
    cfg = synth.Config("halves", layers=4, kv_heads=H, head_dim=128, tokens=700, dtype=dtype, n_codewords=16)
    Ks, Vs, lo_l, lg_l = build_stack(cfg, rht_group=rht_group)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    T = cfg.tokens
    sk, sv = torch.cuda.Stream(), torch.cuda.Stream()
    sk.wait_stream(torch.cuda.current_stream()); sv.wait_stream(torch.cuda.current_stream())
    enc, dec = [], []
    Kp = Vp = None
    for l, lg in enumerate(lg_l):                        # encode: K chain on sk, V chain on sv
        kc, ks = lg.alloc_codes(T)
        vc, vs = lg.alloc_codes(T)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        wk, wv = lg.alloc_workspace(T), lg.alloc_workspace(T)
        B.aquakv_encode_keys(lg, T, Ks[l], Kp, kc, ks, Kh, wk, stream=sk)
        ev = torch.cuda.Event(); ev.record(sk)
        sv.wait_event(ev)
        B.aquakv_encode_values(lg, T, Vs[l], Vp, Kh, vc, vs, Vh, wv, stream=sv)
        enc.append((kc, ks, vc, vs, Kh, Vh, wk, wv))
        Kp, Vp = Kh, Vh
    sk.synchronize(); sv.synchronize()
    for l, (kc, ks, vc, vs, Kh, Vh, _, _) in enumerate(enc):
        g = out[l]
        assert torch.equal(kc, g["k_codes"]) and torch.equal(ks, g["k_scales"]) and torch.equal(bits(Kh), bits(g["Khat"])), l
        assert torch.equal(vc, g["v_codes"]) and torch.equal(vs, g["v_scales"]) and torch.equal(bits(Vh), bits(g["Vhat"])), l
    Kp = Vp = None
    for l, lg in enumerate(lg_l):                        # decode likewise
        g = out[l]
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        wk, wv = lg.alloc_workspace(T), lg.alloc_workspace(T)
        with torch.cuda.stream(sk):
            B.aquakv_decode_layer(lg, T, g["k_codes"], g["k_scales"], None, None, Kp, None, Kh, None, wk, stream=sk)
        ev = torch.cuda.Event(); ev.record(sk)
        sv.wait_event(ev)
        B.aquakv_decode_values(lg, T, g["v_codes"], g["v_scales"], Vp, Kh, Vh, wv, stream=sv)
        dec.append((Kh, Vh, wk, wv))
        Kp, Vp = Kh, Vh
    sk.synchronize(); sv.synchronize()
    for l, (Kh, Vh, _, _) in enumerate(dec):
        assert torch.equal(bits(Kh), bits(out[l]["Khat"])) and torch.equal(bits(Vh), bits(out[l]["Vhat"])), l


# ------------------------------------------------------------------ rotation groups of 1024 across the heads
@pytest.mark.parametrize("dtype,n", [("bf16", 16), ("bf16", 64), ("fp32", 16), ("bf16", 256)])
def test_rotation_group_1024_across_heads(B, dtype, n):
    """rht_group = kv_heads * head_dim (the grouping of the paper's experiments): one rotation and one scale per
    token.  Every stage teacher-forced against the oracle, closed loop, row-count independence, scores."""
    print(f"case group 1024 dtype={dtype} n={n}", flush=True)
    H, T = 8, 333
    cfg = synth.Config("wide", layers=3, kv_heads=H, head_dim=128, tokens=T, dtype=dtype, n_codewords=n)
    Ks, Vs, lo_l, lg_l = build_stack(cfg, rht_group=H * 128)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    for l in range(cfg.layers):
        g, lg = out[l], lg_l[l]
        assert g["k_scales"].shape == (T, 1) and g["k_codes"].shape == (T, H, 16 * (n.bit_length() - 1) // 2)
        for rep in check_layer_against_oracle(B, lo_l[l], lg, Ks[l], Vs[l], g):
            print(f"   layer {l}: {rep}", flush=True)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_decode_layer(lg, T, g["k_codes"], g["k_scales"], g["v_codes"], g["v_scales"], g["Kp"], g["Vp"], Kh, Vh,
                              lg.alloc_workspace(T))
        sync()
        assert torch.equal(bits(Kh), bits(g["Khat"])) and torch.equal(bits(Vh), bits(g["Vhat"]))
        r0, r1 = 57, 121
        cut = lambda t: None if t is None else t[r0:r1].contiguous()
        Kh2, Vh2 = lg.alloc_kv(r1 - r0), lg.alloc_kv(r1 - r0)
        B.aquakv_decode_layer(lg, r1 - r0, cut(g["k_codes"]), cut(g["k_scales"]), cut(g["v_codes"]), cut(g["v_scales"]),
                              cut(g["Kp"]), cut(g["Vp"]), Kh2, Vh2, lg.alloc_workspace(r1 - r0))
        sync()
        assert torch.equal(bits(Kh2), bits(g["Khat"][r0:r1])) and torch.equal(bits(Vh2), bits(g["Vhat"][r0:r1]))
    # the 1024-point rotation gaussianises the synthetic outlier channels better than 128 points:
    # layer-0 relative error close to the grid's own (0.109 / 0.030 / 0.0084)
    K0 = U.np64(Ks[0])
    rel = float(np.sum((U.np64(out[0]["Khat"]) - K0) ** 2) / np.sum(K0 ** 2))
    assert abs(rel / {16: 0.109, 64: 0.030, 256: 0.0084}[n] - 1) < 0.12, rel
    # scores of a predicted layer (the folded form does not exist for this grouping)
    g, lg, lo = out[2], lg_l[2], lo_l[2]
    QH, batch, S = 16, 3, 111
    assert B.aquakv_scores_workspace_bytes(lg, batch, QH) == 0
    q = synth.random_queries(batch, QH, 128, seed=3, dtype=dtype, device="cuda")
    scores = torch.empty(batch, QH, S, dtype=torch.float32, device="cuda")
    B.aquakv_decode_attn_scores(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 0.5, scores, None,
                                lg.alloc_workspace(T))
    sync()
    want = O.attn_scores(lo, batch, S, U.np64(q), g["k_codes"].cpu().numpy(), g["k_scales"].cpu().numpy().view(np.float16),
                         U.np64(g["Kp"]), 0.5)
    Kh = np.abs(U.np64(g["Khat"])).reshape(batch, S, H, 128)
    mag = np.stack([np.einsum("bd,btd->bt", np.abs(U.np64(q))[:, qh], Kh[:, :, qh // (QH // H)]) for qh in range(QH)], 1)
    assert np.all(np.abs(U.np64(scores) - want) <= U.RTOL[dtype] * 0.5 * mag + 1e-30)


@pytest.mark.parametrize("quantizer", ["n16", "n64", "n256", "rtn2", "rtn4"])
def test_fused_encoder_for_groups_of_1024_equals_the_stage_calls(B, quantizer):
    """Groups across the heads (Sect. 4.1): the layer-level encode runs predictor and whole-token quantizer in one
    kernel (64 tokens x 8 heads per workgroup, the predictor weights read from a re-tiled copy in the workspace).  It
    must give, bit for bit, what the stage calls give (aquakv_predict -> fp32 prediction -> aquakv_quantize, the route
    the oracle comparison of test_rotation_group_1024_across_heads teacher-forces), for token counts around the 64-row
    slab and its 32-row halves, with a bias, without the Khat output, and in place."""
    print(f"case fused encoder, groups of 1024, {quantizer}", flush=True)
    H, D = 8, 1024
    kw = dict(rtn_bits=int(quantizer[3:])) if quantizer.startswith("rtn") else {}
    n = 16 if quantizer.startswith("rtn") else int(quantizer[1:])
    gb = torch.Generator().manual_seed(5)
    bk, bv = torch.randn(D, generator=gb) * 0.3, torch.randn(D, generator=gb) * 0.3
    _, lg = U.make_layers(H, "bf16", n, layer_idx=1, w_k=U.random_weights(D, D, 11, 0.7), w_v=U.random_weights(D, 2 * D, 12, 0.7),
                          b_k=bk, b_v=bv, rht_group=1024, **kw)
    for T in (1, 31, 32, 33, 63, 64, 65, 130, 257):
        g = torch.Generator(device="cuda").manual_seed(100 + T)
        mk = lambda: torch.randn(T, H, 128, generator=g, device="cuda").bfloat16()
        K, V, Kp, Vp = mk(), mk(), mk(), mk()
        kc, ks = lg.alloc_codes(T); vc, vs = lg.alloc_codes(T)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        for t in (kc, ks, vc, vs, Kh, Vh):
            t.view(torch.uint8).fill_(0xAB)
        B.aquakv_encode_layer(lg, T, K, V, Kp, Vp, kc, ks, vc, vs, Kh, Vh, lg.alloc_workspace(T))
        # the same through the stage calls
        P = torch.empty(T, D, dtype=torch.float32, device="cuda")
        kc2, ks2 = lg.alloc_codes(T); vc2, vs2 = lg.alloc_codes(T)
        Kh2, Vh2 = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_predict(lg, B.AQUAKV_KEY, T, Kp, None, P)
        B.aquakv_quantize(lg, B.AQUAKV_KEY, T, K, P, kc2, ks2, Kh2)
        B.aquakv_predict(lg, B.AQUAKV_VALUE, T, Vp, Kh2, P)
        B.aquakv_quantize(lg, B.AQUAKV_VALUE, T, V, P, vc2, vs2, Vh2)
        sync()
        for name, a, b in (("k_codes", kc, kc2), ("k_scales", ks, ks2), ("v_codes", vc, vc2), ("v_scales", vs, vs2)):
            assert torch.equal(a, b), (T, name)
        assert torch.equal(bits(Kh), bits(Kh2)) and torch.equal(bits(Vh), bits(Vh2)), T
        # without the reconstructions as outputs (the keys' then go through the workspace), and in place
        kc3, ks3 = lg.alloc_codes(T); vc3, vs3 = lg.alloc_codes(T)
        B.aquakv_encode_layer(lg, T, K, V, Kp, Vp, kc3, ks3, vc3, vs3, None, None, lg.alloc_workspace(T))
        K2, V2 = K.clone(), V.clone()
        kc4, ks4 = lg.alloc_codes(T); vc4, vs4 = lg.alloc_codes(T)
        B.aquakv_encode_layer(lg, T, K2, V2, Kp, Vp, kc4, ks4, vc4, vs4, K2, V2, lg.alloc_workspace(T))
        sync()
        assert torch.equal(kc3, kc) and torch.equal(ks3, ks) and torch.equal(vc3, vc) and torch.equal(vs3, vs), T
        assert torch.equal(kc4, kc) and torch.equal(vs4, vs) and torch.equal(bits(K2), bits(Kh)) and torch.equal(bits(V2), bits(Vh)), T
    print("   token counts 1 .. 257: codes, scales and reconstructions equal those of the stage calls bit for bit", flush=True)


@pytest.mark.parametrize("H,T,quantizer", [(8, 8200, "n16"), (8, 8449, "rtn2"), (6, 11010, "n64"), (16, 4100, "n256"),
                                           (4, 16390, "rtn4"), (8, 16384, "n64"),
                                           # rotation groups of 1024: decode and scores on the large tile (the encoder has its own kernel)
                                           (8, 8200, "n16-g1024"), (8, 8449, "n256-g1024"), (8, 8300, "n64-g1024"),
                                           (8, 8200, "rtn2-g1024")])
def test_two_head_tiles_give_the_bits_of_one_head_tiles(B, H, T, quantizer):
    """Encode, decode and the scoring call switch to tiles of 256 tokens x two heads once that costs no extra round
    over the CUs (the token counts here; short ranges stay on tiles of one head).  The large tile must give the codes,
    scales and reconstructions of the small tile bit for bit (short ranges of the same rows; ragged last tile,
    workgroup counts that are and are not a multiple of the 8 XCDs, with bias, all five quantizers, without the
    reconstruction outputs and in place), decode must reproduce the encoder's reconstructions, the scores must be
    those of the small tile, plain and with the rotary embedding, and the encoder is checked against the oracle
    on sampled rows (grids)."""
    print(f"case two-head tiles H={H} T={T} {quantizer}", flush=True)
    D = H * 128
    wide = quantizer.endswith("-g1024")
    quantizer = quantizer.split("-")[0]
    kw = dict(rtn_bits=int(quantizer[3:])) if quantizer.startswith("rtn") else {}
    if wide:
        kw["rht_group"] = 1024
    n = 16 if quantizer.startswith("rtn") else int(quantizer[1:])
    gb = torch.Generator().manual_seed(6)
    bk, bv = torch.randn(D, generator=gb) * 0.3, torch.randn(D, generator=gb) * 0.3
    lo, lg = U.make_layers(H, "bf16", n, layer_idx=1, w_k=U.random_weights(D, D, 21, 0.7),
                           w_v=U.random_weights(D, 2 * D, 22, 0.7), b_k=bk, b_v=bv, **kw)
    g = torch.Generator(device="cuda").manual_seed(300 + T)
    mk = lambda: torch.randn(T, H, 128, generator=g, device="cuda").bfloat16()
    K, V, Kp, Vp = mk(), mk(), mk(), mk()
    kc, ks = lg.alloc_codes(T); vc, vs = lg.alloc_codes(T)
    Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
    ws = lg.alloc_workspace(T)
    B.aquakv_encode_layer(lg, T, K, V, Kp, Vp, kc, ks, vc, vs, Kh, Vh, ws)
    sync()
    out = dict(k_codes=kc, k_scales=ks, v_codes=vc, v_scales=vs, Khat=Kh, Vhat=Vh, Kp=Kp, Vp=Vp)
    if not kw:               # (the round-to-nearest encoder has its oracle comparison in test_gpu_rtn_backbone.py, the
                             # one for groups of 1024 in test_rotation_group_1024_across_heads)
        for rep in check_layer_against_oracle(B, lo, lg, K, V, out, rows=sampled_rows(T, 48, 4)):
            print(f"   {rep}", flush=True)
    Kd, Vd = lg.alloc_kv(T), lg.alloc_kv(T)
    for t in (Kd, Vd):
        t.view(torch.uint8).fill_(0xAB)
    B.aquakv_decode_layer(lg, T, kc, ks, vc, vs, Kp, Vp, Kd, Vd, ws)
    sync()
    assert torch.equal(bits(Kd), bits(Kh)) and torch.equal(bits(Vd), bits(Vh))
    # the encoder on short ranges of the same rows (small tile): same codes, scales and reconstructions
    for r0, r1 in [(0, 300), (T - 259, T)]:
        m = r1 - r0
        cut = lambda x: x[r0:r1].contiguous()
        kc2, ks2 = lg.alloc_codes(m); vc2, vs2 = lg.alloc_codes(m)
        Kh2, Vh2 = lg.alloc_kv(m), lg.alloc_kv(m)
        B.aquakv_encode_layer(lg, m, cut(K), cut(V), cut(Kp), cut(Vp), kc2, ks2, vc2, vs2, Kh2, Vh2, lg.alloc_workspace(m))
        sync()
        for name, a, b in (("k_codes", kc, kc2), ("k_scales", ks, ks2), ("v_codes", vc, vc2), ("v_scales", vs, vs2)):
            assert torch.equal(a[r0:r1], b), (r0, name)
        assert torch.equal(bits(Kh[r0:r1]), bits(Kh2)) and torch.equal(bits(Vh[r0:r1]), bits(Vh2)), r0
    # without the reconstructions as outputs, and in place
    kc3, ks3 = lg.alloc_codes(T); vc3, vs3 = lg.alloc_codes(T)
    B.aquakv_encode_layer(lg, T, K, V, Kp, Vp, kc3, ks3, vc3, vs3, None, None, ws)
    K2, V2 = K.clone(), V.clone()
    kc4, ks4 = lg.alloc_codes(T); vc4, vs4 = lg.alloc_codes(T)
    B.aquakv_encode_layer(lg, T, K2, V2, Kp, Vp, kc4, ks4, vc4, vs4, K2, V2, lg.alloc_workspace(T))
    sync()
    assert torch.equal(kc3, kc) and torch.equal(ks3, ks) and torch.equal(vc3, vc) and torch.equal(vs3, vs)
    assert torch.equal(kc4, kc) and torch.equal(vs4, vs) and torch.equal(bits(K2), bits(Kh)) and torch.equal(bits(V2), bits(Vh))
    # scores: the whole range (large tile) against short ranges of the same rows (small tile), bit for bit
    QH = 2 * H
    batch, S = (2, T // 2) if T % 2 == 0 else (1, T)
    q = synth.random_queries(batch, QH, 128, seed=17, dtype="bf16", device="cuda")
    cos, sin = O.rope_tables(S, 128, base=500000.0)
    cos_d = torch.from_numpy(cos.astype(np.float32)).cuda()
    sin_d = torch.from_numpy(sin.astype(np.float32)).cuda()
    plain = torch.full((batch, QH, S), float("nan"), dtype=torch.float32, device="cuda")
    roped = torch.full((batch, QH, S), float("nan"), dtype=torch.float32, device="cuda")
    Ko = lg.alloc_kv(T)
    B.aquakv_decode_attn_scores(lg, batch, S, QH, kc, ks, Kp, q, 0.125, plain, Ko, ws)
    B.aquakv_decode_attn_scores_rope(lg, batch, S, QH, kc, ks, Kp, q, cos_d, sin_d, 0.125, roped, None, ws)
    sync()
    assert torch.equal(bits(Ko), bits(Kh))
    assert torch.isfinite(plain).all() and torch.isfinite(roped).all()
    for b, t0, t1 in [(0, 0, 300), (batch - 1, S - 259, S)]:
        r0, r1, n_rows = b * S + t0, b * S + t1, t1 - t0
        cut = lambda x: x[r0:r1].contiguous()
        sp = torch.empty(1, QH, n_rows, dtype=torch.float32, device="cuda")
        B.aquakv_decode_attn_scores(lg, 1, n_rows, QH, cut(kc), cut(ks), cut(Kp), q[b:b + 1].contiguous(), 0.125, sp, None,
                                    lg.alloc_workspace(n_rows))
        sync()
        assert torch.equal(sp[0], plain[b, :, t0:t1]), (b, t0)
        if t0 == 0:                                   # positions of a short range start at 0
            sr = torch.empty(1, QH, n_rows, dtype=torch.float32, device="cuda")
            B.aquakv_decode_attn_scores_rope(lg, 1, n_rows, QH, cut(kc), cut(ks), cut(Kp), q[b:b + 1].contiguous(),
                                             cos_d[:n_rows].contiguous(), sin_d[:n_rows].contiguous(), 0.125, sr, None,
                                             lg.alloc_workspace(n_rows))
            sync()
            assert torch.equal(sr[0], roped[b, :, t0:t1]), (b, t0)
    # and against the definition on the decoded keys, sampled rows
    rows = sampled_rows(T, 48, 8)
    k64 = np.repeat(U.np64(Kh[rows]), 2, axis=1)
    qb = U.np64(q)[(rows // S).cpu().numpy()]                                   # the query of each row's sequence
    want = 0.125 * np.einsum("tqd,tqd->tq", qb, k64)
    mag = 0.125 * np.einsum("tqd,tqd->tq", np.abs(qb), np.abs(k64))
    got = U.np64(plain.permute(0, 2, 1).reshape(T, QH)[rows])
    assert np.all(np.abs(got - want) <= U.RTOL["bf16"] * mag + 1e-30)


# ------------------------------------------------------------------ fused dequant + q.k
@pytest.mark.parametrize("dtype,n,with_pred", [("fp32", 16, True), ("bf16", 16, True), ("bf16", 64, False),
                                               ("bf16", 16, False)])
def test_attn_scores(B, dtype, n, with_pred):
    print(f"case scores dtype={dtype} n={n} pred={with_pred}", flush=True)
    H, QH, batch, S = 8, 32, 3, 150
    cfg = synth.Config("sc", layers=2, kv_heads=H, head_dim=128, tokens=batch * S, dtype=dtype, n_codewords=n)
    Ks, Vs, lo_l, lg_l = build_stack(cfg)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    l = 1 if with_pred else 0
    g, lg, lo = out[l], lg_l[l], lo_l[l]
    q = synth.random_queries(batch, QH, 128, seed=77, dtype=dtype, device="cuda")
    scores = torch.empty(batch, QH, S, dtype=torch.float32, device="cuda")
    Kout = lg.alloc_kv(cfg.tokens)
    B.aquakv_decode_attn_scores(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 0.125, scores, Kout,
                                lg.alloc_workspace(cfg.tokens))
    sync()
    assert torch.equal(bits(Kout), bits(g["Khat"]))
    kp = None if g["Kp"] is None else U.np64(g["Kp"])
    want = O.attn_scores(lo, batch, S, U.np64(q), g["k_codes"].cpu().numpy(), g["k_scales"].cpu().numpy().view(np.float16),
                         kp, 0.125)
    # tolerance relative to sum_d |q_d| |k_d| of the GPU's own keys
    Kh = np.abs(U.np64(g["Khat"])).reshape(batch, S, H, 128)
    mag = np.stack([np.einsum("bd,btd->bt", np.abs(U.np64(q))[:, qh], Kh[:, :, qh // (QH // H)]) for qh in range(QH)], 1)
    err = np.abs(U.np64(scores) - want)
    rtol = U.RTOL[dtype]
    assert np.all(err <= rtol * 0.125 * mag + 1e-30), float(np.max(err / (0.125 * mag + 1e-30)))
    print(f"   worst score error / (sum|q||k|) = {float(np.max(err / (0.125 * mag + 1e-30))):.3g}", flush=True)
    # without Khat_out the scores are the same bits, whatever the size of the workspace (the folded form is a
    # call of its own: a large workspace must not switch the arithmetic)
    for ws2 in ((torch.empty(16, dtype=torch.uint8, device="cuda") if dtype == "bf16" else lg.alloc_workspace(cfg.tokens)),
                torch.empty(max(B.aquakv_scores_workspace_bytes(lg, batch, QH), lg.alloc_workspace(cfg.tokens).numel()) + 4096,
                            dtype=torch.uint8, device="cuda")):
        s2 = torch.empty_like(scores)
        B.aquakv_decode_attn_scores(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 0.125, s2, None, ws2)
        sync()
        assert torch.equal(s2, scores)
    # folded form (predictor folded into the query): same definition, unrounded keys
    need = B.aquakv_scores_workspace_bytes(lg, batch, QH)
    assert (need > 0) == (dtype == "bf16" and with_pred)
    if need:
        s3 = torch.full_like(scores, float("nan"))
        B.aquakv_decode_attn_scores_folded(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 0.125, s3,
                                           lg.alloc_scores_workspace(batch, QH))
        sync()
        err3 = np.abs(U.np64(s3) - want)
        assert np.all(err3 <= rtol * 0.125 * mag + 1e-30), float(np.max(err3 / (0.125 * mag + 1e-30)))
        assert not torch.equal(s3, scores)          # it really was the other kernel
        print(f"   folded: worst score error / (sum|q||k|) = {float(np.max(err3 / (0.125 * mag + 1e-30))):.3g}", flush=True)


@pytest.mark.parametrize("n,QH,batch,S,bias", [(16, 24, 2, 100, True), (64, 32, 1, 1000, False), (256, 8, 3, 33, True),
                                              (16, 16, 5, 31, False), (16, 64, 2, 70, True), (64, 40, 1, 130, False)])
def test_folded_scores_against_definition(B, n, QH, batch, S, bias):
    """aquakv_decode_attn_scores_folded against the oracle's plain definition
    (decode the keys, round them to storage, dot with q): query heads per kv head 1..4 (one pass), 5 and 8
    (two passes), all three grids, predictor bias, ragged last tile, sequences shorter than one tile."""
    print(f"case folded scores n={n} QH={QH} batch={batch} S={S} bias={bias}", flush=True)
    H = 8
    cfg = synth.Config("fold", layers=2, kv_heads=H, head_dim=128, tokens=batch * S, dtype="bf16", n_codewords=n)
    Ks, Vs, lo_l, lg_l = build_stack(cfg, bias=bias)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    g, lg, lo = out[1], lg_l[1], lo_l[1]
    q = synth.random_queries(batch, QH, 128, seed=5, dtype="bf16", device="cuda")
    need = B.aquakv_scores_workspace_bytes(lg, batch, QH)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    scores = torch.full((batch, QH, S), float("nan"), dtype=torch.float32, device="cuda")
    B.aquakv_decode_attn_scores_folded(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 0.25, scores, ws)
    sync()
    want = O.attn_scores(lo, batch, S, U.np64(q), g["k_codes"].cpu().numpy(), g["k_scales"].cpu().numpy().view(np.float16),
                         U.np64(g["Kp"]), 0.25)
    Kh = np.abs(U.np64(g["Khat"])).reshape(batch, S, H, 128)
    mag = np.stack([np.einsum("bd,btd->bt", np.abs(U.np64(q))[:, qh], Kh[:, :, qh // (QH // H)]) for qh in range(QH)], 1)
    err = np.abs(U.np64(scores) - want)
    worst = float(np.max(err / (0.25 * mag + 1e-30)))
    assert np.all(err <= U.RTOL["bf16"] * 0.25 * mag + 1e-30), worst
    print(f"   worst score error / (sum|q||k|) = {worst:.3g}", flush=True)
    # a second call into the same workspace with other queries (fewer heads) leaves no residue
    QH2 = 8
    q2 = synth.random_queries(batch, QH2, 128, seed=6, dtype="bf16", device="cuda")
    sc2 = torch.empty(batch, QH2, S, dtype=torch.float32, device="cuda")
    B.aquakv_decode_attn_scores_folded(lg, batch, S, QH2, g["k_codes"], g["k_scales"], g["Kp"], q2, 0.25, sc2, ws)
    sync()
    want2 = O.attn_scores(lo, batch, S, U.np64(q2), g["k_codes"].cpu().numpy(),
                          g["k_scales"].cpu().numpy().view(np.float16), U.np64(g["Kp"]), 0.25)
    mag2 = np.stack([np.einsum("bd,btd->bt", np.abs(U.np64(q2))[:, qh], Kh[:, :, qh]) for qh in range(QH2)], 1)
    assert np.all(np.abs(U.np64(sc2) - want2) <= U.RTOL["bf16"] * 0.25 * mag2 + 1e-30)


@pytest.mark.parametrize("dtype,n,with_pred", [("bf16", 16, True), ("bf16", 64, False), ("fp32", 16, True)])
def test_attn_scores_with_rotary_embedding(B, dtype, n, with_pred):
    """aquakv_decode_attn_scores_rope: keys cached before the rotary embedding are rotated by their position
    after decoding (fused kernel with predictor, stand-alone kernel for layer 0 and fp32); Khat_out stays unrotated."""
    print(f"case rope scores dtype={dtype} n={n} pred={with_pred}", flush=True)
    H, QH, batch, S = (8, 32, 2, 300) if dtype == "bf16" else (2, 8, 2, 70)
    cfg = synth.Config("rope", layers=2, kv_heads=H, head_dim=128, tokens=batch * S, dtype=dtype, n_codewords=n)
    Ks, Vs, lo_l, lg_l = build_stack(cfg)
    out = run_gpu_layers(B, cfg, lg_l, Ks, Vs)
    l = 1 if with_pred else 0
    g, lg, lo = out[l], lg_l[l], lo_l[l]
    q = synth.random_queries(batch, QH, 128, seed=78, dtype=dtype, device="cuda")
    cos, sin = O.rope_tables(S, 128, base=500000.0)
    cos_d = torch.from_numpy(cos.astype(np.float32)).cuda()
    sin_d = torch.from_numpy(sin.astype(np.float32)).cuda()
    scores = torch.full((batch, QH, S), float("nan"), dtype=torch.float32, device="cuda")
    Kout = lg.alloc_kv(cfg.tokens)
    B.aquakv_decode_attn_scores_rope(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, cos_d, sin_d, 0.125, scores,
                                     Kout, lg.alloc_workspace(cfg.tokens))
    sync()
    assert torch.equal(bits(Kout), bits(g["Khat"]))                      # unrotated keys out
    kp = None if g["Kp"] is None else U.np64(g["Kp"])
    want = O.attn_scores(lo, batch, S, U.np64(q), g["k_codes"].cpu().numpy(), g["k_scales"].cpu().numpy().view(np.float16),
                         kp, 0.125, rope=(cos, sin))
    plain = O.attn_scores(lo, batch, S, U.np64(q), g["k_codes"].cpu().numpy(), g["k_scales"].cpu().numpy().view(np.float16),
                          kp, 0.125)
    assert np.max(np.abs(want - plain)[:, :, 1:]) > 0.1                   # the rotation matters in this test
    Kh = np.abs(U.np64(g["Khat"])).reshape(batch, S, H, 128)
    # a rotation mixes |k_d| and |k_{d+64}|: bound each rotated magnitude by their sum
    Kh = Kh + np.concatenate([Kh[..., 64:], Kh[..., :64]], axis=-1)
    mag = np.stack([np.einsum("bd,btd->bt", np.abs(U.np64(q))[:, qh], Kh[:, :, qh // (QH // H)]) for qh in range(QH)], 1)
    err = np.abs(U.np64(scores) - want)
    rtol = U.RTOL[dtype]
    worst = float(np.max(err / (0.125 * mag + 1e-30)))
    assert np.all(err <= rtol * 0.125 * mag + 1e-30), worst
    print(f"   worst score error / (sum|q||k|) = {worst:.3g}", flush=True)
    # position 0 is the identity: the first token of every sequence scores as without rotation
    s0 = torch.empty_like(scores)
    small = torch.empty(16, dtype=torch.uint8, device="cuda") if dtype == "bf16" and with_pred else lg.alloc_workspace(cfg.tokens)
    B.aquakv_decode_attn_scores(lg, batch, S, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 0.125, s0, None, small)
    sync()
    assert torch.equal(s0[:, :, 0], scores[:, :, 0])


# ------------------------------------------------------------------ full sizes, sampled rows
def sampled_rows(T, n, seed):
    """Seeded sample of token rows that always includes the first / last rows and both sides
    of workgroup-tile boundaries (tiles are 256 rows)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    fixed = [0, 1, 255, 256, 257, T // 2, T - 257, T - 256, T - 2, T - 1]
    extra = rng.choice(T, size=n - len(fixed), replace=False).tolist()
    return torch.tensor(sorted(set(fixed + extra)), device="cuda")


def stream_layers(cfg, n_layers, n_per_layer, device="cuda"):
    """Layer-by-layer generator on the GPU (as bench.py does): yields (l, K, V, oracle layer, gpu layer)."""
    st = synth.KVStream(cfg, device=device, work=torch.float32)
    for l in range(n_layers):
        K, V = st.next()
        if l == 0:
            lo, lg = U.make_layers(cfg.kv_heads, cfg.dtype, n_per_layer[l], layer_idx=l)
        else:
            wk, wv = synth.analytic_predictors(st, l)
            lo, lg = U.make_layers(cfg.kv_heads, cfg.dtype, n_per_layer[l], layer_idx=l, w_k=wk, w_v=wv)
        yield l, K.contiguous(), V.contiguous(), lo, lg


@pytest.mark.parametrize("name,T,n_per_layer", [
    ("llama3.2-3b bench shape", 8192, [16, 16, 16]),
    ("llama3.1-8b shape, 2-bit (the headline workload of bench.py)", 32768, [16, 16, 16]),
    ("llama3.1-8b shape, 3-bit", 32768, [64, 64]),
    ("llama3.1-8b shape, 4-bit", 32768, [256, 256]),
    ("llama3.1-70b shape, mixed 2/3-bit", 131072, [16, 64, 16]),
])
def test_full_size_layers_on_sampled_rows(B, name, T, n_per_layer):
    """The launch configuration bench.py times (all rows of a layer in one call), checked on a
    seeded sample of rows: tokens are independent, so the oracle can follow single rows exactly."""
    print(f"case full size: {name} T={T}", flush=True)
    cfg = synth.Config(name, layers=len(n_per_layer), kv_heads=8, head_dim=128, tokens=T, dtype="bf16")
    rows = sampled_rows(T, 160, 5)
    Kp = Vp = None
    kept = dict(lo=[], lg=[], K=[], V=[], out=[])
    for l, K, V, lo, lg in stream_layers(cfg, len(n_per_layer), n_per_layer):
        kc, ks = lg.alloc_codes(T)
        vc, vs = lg.alloc_codes(T)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        ws = lg.alloc_workspace(T)
        B.aquakv_encode_layer(lg, T, K, V, Kp, Vp, kc, ks, vc, vs, Kh, Vh, ws)
        sync()
        g = dict(k_codes=kc, k_scales=ks, v_codes=vc, v_scales=vs, Khat=Kh, Vhat=Vh, Kp=Kp, Vp=Vp)
        for name, item in (("lo", lo), ("lg", lg), ("K", K), ("V", V), ("out", g)):
            kept[name].append(item)
        for rep in check_layer_against_oracle(B, lo, lg, K, V, g, rows=rows):
            print(f"   layer {l}: {rep}", flush=True)
        Kd, Vd = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_decode_layer(lg, T, kc, ks, vc, vs, Kp, Vp, Kd, Vd, ws)
        sync()
        assert torch.equal(bits(Kd), bits(Kh)) and torch.equal(bits(Vd), bits(Vh))
        # the decode sweep in the form bench.py times: the scoring call with Khat_out is the key half of decode,
        # aquakv_decode_values the value half; same bits, and the scores are q . Khat on the sampled rows
        QH = 64 if T == 131072 else 24
        q = synth.random_queries(1, QH, 128, seed=9 + l, dtype="bf16", device="cuda")
        scores = torch.empty(1, QH, T, dtype=torch.float32, device="cuda")
        Kd2, Vd2 = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_decode_attn_scores(lg, 1, T, QH, kc, ks, Kp, q, 0.088388, scores, Kd2, ws)
        B.aquakv_decode_values(lg, T, vc, vs, Vp, Kd2, Vd2, ws)
        sync()
        assert torch.equal(bits(Kd2), bits(Kh)) and torch.equal(bits(Vd2), bits(Vh))
        k64 = np.repeat(U.np64(Kh[rows]), QH // 8, axis=1)                       # [rows, QH, 128]
        want = 0.088388 * np.einsum("qd,tqd->qt", U.np64(q)[0], k64)
        mag = 0.088388 * np.einsum("qd,tqd->qt", np.abs(U.np64(q)[0]), np.abs(k64))
        got = U.np64(scores[0][:, rows])
        assert np.all(np.abs(got - want) <= U.RTOL["bf16"] * mag + 1e-30), float(np.max(np.abs(got - want) / (mag + 1e-30)))
        # the value half with the attention output (soft-max of those scores inside): same values, and the output is
        # the oracle's soft-max-weighted sum over the values the call wrote (every output depends on all rows)
        out = torch.empty(1, QH, 128, dtype=torch.float32, device="cuda")
        Vd3 = lg.alloc_kv(T)
        B.aquakv_decode_values_attend(lg, 1, T, QH, vc, vs, Vp, Kd2, scores, Vd3, out, None, lg.alloc_weighted_workspace(1, T, QH))
        sync()
        assert torch.equal(bits(Vd3), bits(Vh))
        p_rows = O.softmax_rows(U.np64(scores))[0]
        v64 = U.np64(Vh)
        own = np.stack([p_rows[qh] @ v64[:, qh // (QH // 8)] for qh in range(QH)])
        mag_v = np.stack([p_rows[qh] @ np.abs(v64[:, qh // (QH // 8)]) for qh in range(QH)])
        err_v = np.abs(U.np64(out)[0] - own)
        assert np.all(err_v <= 3e-5 * mag_v), float(np.max(err_v / mag_v))
        del v64
        # properties that hold at any size: every scale is a finite non-negative fp16, the relative
        # reconstruction error of the whole tensor is what the grid and the predictor allow
        s = ks.view(torch.float16).float()
        assert torch.isfinite(s).all() and (s >= 0).all()
        rel = ((Kh.float() - K.float()).pow(2).sum() / K.float().pow(2).sum()).item()
        bound = {16: 0.13, 64: 0.04, 256: 0.012}[n_per_layer[l]] if l == 0 else {16: 0.06, 64: 0.02, 256: 0.003}[n_per_layer[l]]
        print(f"   layer {l}: relative reconstruction error of the keys {rel:.5f} (bound {bound})", flush=True)
        assert rel < bound, (l, rel)
        Kp, Vp = Kh, Vh
    # free-running: the oracle follows the sampled rows through all layers on its own reconstructions; every
    # disagreement with the library's codes and scales must have a cause (tie, or the measured difference of inputs)
    for l, which, rep in free_run_layers(B, kept["lo"], kept["lg"], kept["K"], kept["V"], kept["out"], rows=rows):
        print(f"   free-run layer {l} {which}: {rep}", flush=True)
        assert rep.other == 0, f"layer {l} {which}: {rep}"


def test_folded_scores_at_the_full_decode_read_shape(B):
    """64 sequences x 16384 cached tokens, 32 query heads (the launch configuration of `bench.py --config
    decode-read`: 32 tiles per workgroup): the folded scoring call against the oracle on sampled (sequence, token)
    pairs.  The oracle scores any codes, so the cache content is drawn directly (random codes, scales, Khat_prev)."""
    print("case folded scores, full decode-read shape", flush=True)
    batch, S, H, QH, n = 64, 16384, 8, 32, 16
    T = batch * S
    gen = torch.Generator(device="cuda").manual_seed(synth.BASE_SEED + 404)
    wk = U.random_weights(1024, 1024, 7, 0.7)
    lo, lg = U.make_layers(H, "bf16", n, layer_idx=3, w_k=wk, w_v=U.random_weights(1024, 2048, 8, 0.7))
    Kprev = torch.randn(T, H, 128, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    kc, ks = lg.alloc_codes(T)
    kc.copy_(torch.randint(0, 256, kc.shape, generator=gen, device="cuda", dtype=torch.int32).to(torch.uint8))
    ks.copy_((torch.rand(T, H, generator=gen, device="cuda") * 2 + 0.05).half().view(torch.int16))
    q = synth.random_queries(batch, QH, 128, seed=12, dtype="bf16", device="cuda")
    need = B.aquakv_scores_workspace_bytes(lg, batch, QH)
    assert need > 0
    scores = torch.full((batch, QH, S), float("nan"), dtype=torch.float32, device="cuda")
    B.aquakv_decode_attn_scores_folded(lg, batch, S, QH, kc, ks, Kprev, q, 0.0883883, scores,
                                       torch.empty(need, dtype=torch.uint8, device="cuda"))
    sync()
    assert torch.isfinite(scores).all()
    rng = np.random.Generator(np.random.PCG64(91))
    worst = 0.0
    for b in (0, 17, batch - 1):
        ts = np.unique(np.concatenate([[0, 31, 32, 1023, 1024, S - 33, S - 1], rng.choice(S, 48, replace=False)]))
        sel = torch.from_numpy(b * S + ts).cuda()
        want = O.attn_scores(lo, 1, len(ts), U.np64(q[b:b + 1]), kc[sel].cpu().numpy(), ks[sel].cpu().numpy().view(np.float16),
                             U.np64(Kprev[sel]), 0.0883883)[0]
        got = U.np64(scores[b][:, torch.from_numpy(ts).cuda()])
        Khat, _ = O.decode_layer(lo, kc[sel].cpu().numpy(), ks[sel].cpu().numpy().view(np.float16), kc[sel].cpu().numpy(),
                                 ks[sel].cpu().numpy().view(np.float16), U.np64(Kprev[sel]), U.np64(Kprev[sel]))
        Ka = np.abs(Khat)
        mag = np.stack([np.abs(U.np64(q[b, qh])) @ Ka[:, qh // (QH // H)].T for qh in range(QH)], 0)
        err = np.abs(got - want)
        assert np.all(err <= U.RTOL["bf16"] * 0.0883883 * mag + 1e-30)
        worst = max(worst, float(np.max(err / (0.0883883 * mag + 1e-30))))
    print(f"   worst score error / sum|q||k| = {worst:.2e}", flush=True)


@pytest.mark.parametrize("batch", [8, 64])
def test_decode_read_path_batch_of_long_sequences(B, batch):
    """The decode-phase read path (batched sequences of 16384 cached tokens, 32 query heads on 8 kv
    heads; batch 64 is the full shape of the workload list): fused dequantize + q.k (the definition: prediction
    recomputed, rounded keys scored) against the oracle on sampled (sequence, token) pairs, plus the
    one-new-token-per-sequence append through aquakv_encode_layer."""
    print(f"case decode read path batch={batch}", flush=True)
    S, H, QH, n = 16384, 8, 32, 16
    T = batch * S
    cfg = synth.Config("read-path", layers=2, kv_heads=H, head_dim=128, tokens=T, dtype="bf16")
    outs = []
    Kp = Vp = None
    for l, K, V, lo, lg in stream_layers(cfg, 2, [n, n]):
        kc, ks = lg.alloc_codes(T)
        vc, vs = lg.alloc_codes(T)
        Kh, Vh = lg.alloc_kv(T), lg.alloc_kv(T)
        B.aquakv_encode_layer(lg, T, K, V, Kp, Vp, kc, ks, vc, vs, Kh, Vh, lg.alloc_workspace(T))
        sync()
        outs.append((lo, lg, kc, ks, Kh, Kp, K, V, Vp, vc, vs, Vh))
        Kp, Vp = Kh, Vh
    q = synth.random_queries(batch, QH, 128, seed=9, dtype="bf16", device="cuda")
    for l, (lo, lg, kc, ks, Kh, Kprev, K, V, Vprev, vc, vs, Vh) in enumerate(outs):
        scores = torch.empty(batch, QH, S, dtype=torch.float32, device="cuda")
        B.aquakv_decode_attn_scores(lg, batch, S, QH, kc, ks, Kprev, q, 0.0883883, scores, None, lg.alloc_workspace(T))
        sync()
        rng = np.random.Generator(np.random.PCG64(17 + l))
        for b in (0, 3, batch - 1):
            ts = np.unique(np.concatenate([[0, 255, 256, S - 1], rng.choice(S, 40, replace=False)]))
            sel = torch.from_numpy(b * S + ts).cuda()
            kp = None if Kprev is None else U.np64(Kprev[sel])
            want = O.attn_scores(lo, 1, len(ts), U.np64(q[b:b + 1]), kc[sel].cpu().numpy(),
                                 ks[sel].cpu().numpy().view(np.float16), kp, 0.0883883)[0]
            got = U.np64(scores[b][:, torch.from_numpy(ts).cuda()])
            Ka = np.abs(U.np64(Kh[sel])).reshape(len(ts), H, 128)
            mag = np.stack([np.abs(U.np64(q[b, qh])) @ Ka[:, qh // (QH // H)].T for qh in range(QH)], 0)
            err = np.abs(got - want)
            assert np.all(err <= U.RTOL["bf16"] * 0.0883883 * mag + 1e-30)
            print(f"   layer {l} seq {b}: worst score error / sum|q||k| = "
                  f"{float(np.max(err / (0.0883883 * mag + 1e-30))):.2e}", flush=True)
    # append: one new token per sequence = an encode call with tokens = batch; it must give the
    # same bytes as the rows had inside the big call (row-count independence of the predictor)
    lo, lg, kc, ks, Kh, Kprev, K, V, Vprev, vc, vs, Vh = outs[1]
    new = torch.arange(batch, device="cuda") * S + (S - 1)
    cut = lambda t: t[new].contiguous()
    kc2, ks2 = lg.alloc_codes(batch)
    vc2, vs2 = lg.alloc_codes(batch)
    Kh2, Vh2 = lg.alloc_kv(batch), lg.alloc_kv(batch)
    B.aquakv_encode_layer(lg, batch, cut(K), cut(V), cut(Kprev), cut(Vprev), kc2, ks2, vc2, vs2, Kh2, Vh2,
                          lg.alloc_workspace(batch))
    sync()
    assert torch.equal(kc2, cut(kc)) and torch.equal(ks2, cut(ks)) and torch.equal(vc2, cut(vc))
    assert torch.equal(bits(Kh2), bits(cut(Kh))) and torch.equal(bits(Vh2), bits(cut(Vh)))


def test_group_1024_at_the_bench_shape(B):
    """Rotation groups of 1024 at 8192 tokens (the launch shape of `bench.py --rht-group 1024`): the fused decode,
    scores and attention forms reproduce what the (unfused) encoder reconstructed, bit for bit, and the scores and
    sums are those of the tensors written."""
    print("case group 1024 at 8192 tokens", flush=True)
    H, T, QH = 8, 8192, 24
    cfg = synth.Config("wide8k", layers=2, kv_heads=H, head_dim=128, tokens=T, dtype="bf16", n_codewords=16)
    Ks, Vs, lo_l, lg_l = build_stack(cfg, rht_group=H * 128)
    g = run_gpu_layers(B, cfg, lg_l, Ks, Vs)[1]
    lg = lg_l[1]
    ws = lg.alloc_workspace(T)
    Kd, Vd = lg.alloc_kv(T), lg.alloc_kv(T)
    B.aquakv_decode_layer(lg, T, g["k_codes"], g["k_scales"], g["v_codes"], g["v_scales"], g["Kp"], g["Vp"], Kd, Vd, ws)
    sync()
    assert torch.equal(bits(Kd), bits(g["Khat"])) and torch.equal(bits(Vd), bits(g["Vhat"]))
    q = synth.random_queries(1, QH, 128, seed=4, dtype="bf16", device="cuda")
    scores = torch.empty(1, QH, T, dtype=torch.float32, device="cuda")
    out = torch.empty(1, QH, 128, dtype=torch.float32, device="cuda")
    Kd.zero_(); Vd.zero_()
    B.aquakv_decode_attn_scores(lg, 1, T, QH, g["k_codes"], g["k_scales"], g["Kp"], q, 0.088388, scores, Kd, ws)
    B.aquakv_decode_values_attend(lg, 1, T, QH, g["v_codes"], g["v_scales"], g["Vp"], Kd, scores, Vd, out, None,
                                  lg.alloc_weighted_workspace(1, T, QH))
    sync()
    assert torch.equal(bits(Kd), bits(g["Khat"])) and torch.equal(bits(Vd), bits(g["Vhat"]))
    k64, v64, q64 = U.np64(Kd), U.np64(Vd), U.np64(q)[0]
    want_s = 0.088388 * np.stack([k64[:, qh // 3] @ q64[qh] for qh in range(QH)])
    mag_s = 0.088388 * np.stack([np.abs(k64[:, qh // 3]) @ np.abs(q64[qh]) for qh in range(QH)])
    assert np.all(np.abs(U.np64(scores)[0] - want_s) <= 1e-5 * mag_s + 1e-30)
    p_rows = O.softmax_rows(U.np64(scores))[0]
    own = np.stack([p_rows[qh] @ v64[:, qh // 3] for qh in range(QH)])
    mag_v = np.stack([p_rows[qh] @ np.abs(v64[:, qh // 3]) for qh in range(QH)])
    assert np.all(np.abs(U.np64(out)[0] - own) <= 3e-5 * mag_v)
