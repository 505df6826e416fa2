"""Micro-benchmarks of the single calls of the library, for sizing a deployment and for checking a kernel against its
roofline away from the whole-job benchmark: `python -m paper_2501_19392_amd.microbench <what>`.

  kscan       fused encode / decode / scores and the stand-alone predictor against the predictor's input width K
              (Sect. 3.2 of the AQUA-KV paper: K = d for keys, 2 d for values); K = 128 is launch + epilogue almost alone
  standalone  the backbone quantizer alone (Sect. 2; the first layer, which has no predictor): quantize, dequantize and
              scores from codes, against the bytes they must move
  ceilings    what this GPU sustains on plain streams (fill, copy, read-only reduction): the practical HBM ceiling the
              kernels above are held against, beside the nominal 8 TB/s
  gemm        the bf16 predictor GEMM shapes: the vendor library (torch.nn.functional.linear, a yardstick only, never
              a code path) beside aquakv_predict and the fused decode call
  clock       engine clock and power reported by rocm-smi while fused encode launches run back to back

Every line is one measurement: mean over back-to-back launches between two events on the current stream, inputs
resident in HBM, random normal data (timings do not depend on the values except through the rare full-search pass
of the quantizer).
"""
from __future__ import annotations

import argparse
import subprocess
import sys


def _timeit(torch, fn, reps=20, warm=3):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps                 # microseconds per launch


def _layer(torch, B, synth, n, K, H=8, dev="cuda", seed=0):
    """A predicted key layer with a d x K predictor (K = 0: no predictor)."""
    C = torch.from_numpy(synth.lloyd_codebook(n)).to(dev)
    s = torch.from_numpy(synth.rht_signs(H, 128, 1, "k")).to(dev)
    kw = {}
    if K:
        g = torch.Generator().manual_seed(seed + K)
        kw["w_k"] = (torch.randn(H * 128, K, generator=g) / K ** 0.5 * 0.7).to(torch.bfloat16).to(dev)
    return B.Layer(H, 128, C, s, s, torch.bfloat16, search_table=B.build_search_table(C), **kw)


def kscan(args):
    import torch
    from . import binding as B, synth
    T, H, D, QH, dev = args.tokens, 8, 1024, args.q_heads, "cuda"
    print(f"# kscan: {T} tokens x 8 kv heads x 128, bf16, n = {args.n_codewords}, {QH} query heads; microseconds per launch")
    print("K  predict  fused_decode  fused_encode  fused_scores  decode_TFLOPs  encode_TFLOPs", flush=True)
    for K in (128, 256, 512, 1024, 2048, 4096):
        lay = _layer(torch, B, synth, args.n_codewords, K)
        g = torch.Generator(device=dev).manual_seed(K)
        xp = torch.randn(T, K, generator=g, device=dev).to(torch.bfloat16)
        X = torch.randn(T, H, 128, generator=g, device=dev).to(torch.bfloat16)
        P = torch.empty(T, D, dtype=torch.float32, device=dev)
        kc, ks = lay.alloc_codes(T)
        Kh, ws = lay.alloc_kv(T), lay.alloc_workspace(T)
        q = synth.random_queries(1, QH, 128, seed=1, dtype="bf16", device=dev)
        sc = torch.empty(1, QH, T, dtype=torch.float32, device=dev)
        t_p = _timeit(torch, lambda: B.aquakv_predict(lay, B.AQUAKV_KEY, T, xp, None, P))
        t_e = _timeit(torch, lambda: B.aquakv_encode_keys(lay, T, X, xp, kc, ks, Kh, ws))
        t_d = _timeit(torch, lambda: B.aquakv_decode_layer(lay, T, kc, ks, None, None, xp, None, Kh, None, ws))
        t_s = _timeit(torch, lambda: B.aquakv_decode_attn_scores(lay, 1, T, QH, kc, ks, xp, q, 0.1, sc, Kh, ws))
        fl = 2.0 * T * D * K
        print(f"{K}  {t_p:.1f}  {t_d:.1f}  {t_e:.1f}  {t_s:.1f}  {fl / t_d / 1e6:.0f}  {fl / t_e / 1e6:.0f}", flush=True)


def standalone(args):
    import torch
    from . import binding as B, synth
    H, dev = 8, "cuda"
    print("# standalone: backbone quantizer alone, bf16, 8 kv heads x 128; GB/s = algorithmic bytes / time (fraction of 8 TB/s)")
    for n in (16, 64):
        for T in args.token_list:
            lay = _layer(torch, B, synth, n, 0)
            g = torch.Generator(device=dev).manual_seed(0)
            X = torch.randn(T, H, 128, generator=g, device=dev).to(torch.bfloat16)
            codes, scales = lay.alloc_codes(T)
            Xh = lay.alloc_kv(T)
            cb = lay.code_bytes_per_group + 2              # codes + fp16 scale per group of 128
            q = synth.random_queries(1, 32, 128, 1, "bf16", dev)
            sc = torch.empty(1, 32, T, dtype=torch.float32, device=dev)
            for name, nbytes, fn in (
                    ("quantize (codes + reconstruction)", 256 + 256 + cb, lambda: B.aquakv_quantize(lay, 0, T, X, None, codes, scales, Xh)),
                    ("quantize (codes only)", 256 + cb, lambda: B.aquakv_quantize(lay, 0, T, X, None, codes, scales, None)),
                    ("dequantize", 256 + cb, lambda: B.aquakv_dequantize(lay, 0, T, codes, scales, None, Xh)),
                    ("scores from codes (32 query heads)", cb + 16, lambda: B.aquakv_decode_attn_scores(lay, 1, T, 32, codes, scales, None, q, 1.0, sc, None, None))):
                us = _timeit(torch, fn)
                rate = T * H * nbytes / us / 1e3
                print(f"n={n} T={T} {name}: {us:.1f} us  {rate:.0f} GB/s ({rate / 8000:.3f})", flush=True)


def ceilings(args):
    import torch
    dev = "cuda"
    print("# ceilings: plain streams through torch's own kernels; GB/s counts every byte read and written")
    for mb in (64, 256, 1024, 4096):
        n = mb * (1 << 20) // 4
        x = torch.empty(n, dtype=torch.float32, device=dev)
        y = torch.empty(n, dtype=torch.float32, device=dev)
        gb = mb * 1.048576e-3
        us = _timeit(torch, lambda: x.fill_(1.0), reps=10, warm=1)
        print(f"{mb} MiB fill: {us:.1f} us  {gb / us * 1e6:.0f} GB/s written", flush=True)
        us = _timeit(torch, lambda: y.copy_(x), reps=10, warm=1)
        print(f"{mb} MiB copy: {us:.1f} us  {2 * gb / us * 1e6:.0f} GB/s read + written", flush=True)
        us = _timeit(torch, lambda: torch.sum(x), reps=10, warm=1)
        print(f"{mb} MiB sum: {us:.1f} us  {gb / us * 1e6:.0f} GB/s read", flush=True)
        del x, y


def gemm(args):
    import torch
    from . import binding as B, synth
    dev, D = "cuda", 1024
    print("# gemm: T x K times K x 1024, bf16 in, fp32 accumulate; library = torch.nn.functional.linear (yardstick only)")
    print("T  K  library_us  library_TFLOPs  predict_us  predict_TFLOPs  fused_decode_us  fused_decode_TFLOPs", flush=True)
    for T in args.token_list:
        for K in (1024, 2048):
            lay = _layer(torch, B, synth, 16, K)
            x = torch.randn(T, K, device=dev).to(torch.bfloat16)
            w = torch.randn(D, K, device=dev).to(torch.bfloat16)
            P = torch.empty(T, D, dtype=torch.float32, device=dev)
            kc, ks = lay.alloc_codes(T)
            kc.zero_(); ks.fill_(15360)                    # any valid codes; scale 1.0
            Kh, ws = lay.alloc_kv(T), lay.alloc_workspace(T)
            fl = 2.0 * T * D * K
            t_l = _timeit(torch, lambda: torch.nn.functional.linear(x, w))
            t_p = _timeit(torch, lambda: B.aquakv_predict(lay, B.AQUAKV_KEY, T, x, None, P))
            t_d = _timeit(torch, lambda: B.aquakv_decode_layer(lay, T, kc, ks, None, None, x, None, Kh, None, ws))
            print(f"{T}  {K}  {t_l:.1f}  {fl / t_l / 1e6:.0f}  {t_p:.1f}  {fl / t_p / 1e6:.0f}  {t_d:.1f}  {fl / t_d / 1e6:.0f}", flush=True)


def clock(args):
    # the sampler is started before anything touches the GPU in this process
    sampler = subprocess.Popen(
        ["bash", "-c", "rocm-smi --showclocks --showpower 2>&1 | grep -i 'sclk\\|power' | head -4; sleep 6; "
                       "for i in 1 2 3 4; do rocm-smi --showclocks --showpower 2>&1 | grep -i 'sclk\\|power' | head -4; sleep 1; done"],
        stdout=subprocess.PIPE, text=True)
    import time
    import torch
    from . import binding as B, synth
    T, H, K, dev = args.tokens, 8, 1024, "cuda"
    lay = _layer(torch, B, synth, 16, K)
    xp = torch.randn(T, K, device=dev).to(torch.bfloat16)
    X = torch.randn(T, H, 128, device=dev).to(torch.bfloat16)
    kc, ks = lay.alloc_codes(T)
    Kh, ws = lay.alloc_kv(T), lay.alloc_workspace(T)
    t0 = time.time()
    launches = 0
    while time.time() - t0 < 14.0:
        for _ in range(200):
            B.aquakv_encode_keys(lay, T, X, xp, kc, ks, Kh, ws)
        torch.cuda.synchronize()
        launches += 200
    out, _ = sampler.communicate()
    print(f"# clock: rocm-smi before the load (first lines) and four samples while {launches} fused encode launches "
          f"({T} tokens, K = {K}) ran back to back")
    print(out, flush=True)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("what", choices=["kscan", "standalone", "ceilings", "gemm", "clock"])
    ap.add_argument("--tokens", type=int, default=8192, help="token rows (kscan, clock)")
    ap.add_argument("--token-list", type=lambda s: [int(x) for x in s.split(",")], default=[8192, 32768, 131072],
                    help="token rows, comma separated (standalone, gemm)")
    ap.add_argument("--n-codewords", type=int, default=16)
    ap.add_argument("--q-heads", type=int, default=32)
    args = ap.parse_args(argv)
    {"kscan": kscan, "standalone": standalone, "ceilings": ceilings, "gemm": gemm, "clock": clock}[args.what](args)


if __name__ == "__main__":
    sys.exit(main())
