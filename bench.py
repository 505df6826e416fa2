#!/usr/bin/env python3
"""Benchmark of the AQUA-KV per-layer encode / decode path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic KV shaped like
the Llama-3.1-8B cache (32 layers, 8 KV heads x 128, 32768 tokens, bf16, 2 bits per
value): for every layer `aquakv_encode_layer`, then the decode sweep that also yields
the q.k scores (32 query heads).  Inputs are resident in HBM before the timed region.
The printed JSON line reports tokens/s per layer (tokens * layers / step time), the
roofline position of the dominant kernel (the fused bf16 MFMA predictor + quantizer
kernel) from HIP events, one roofline entry per stage (`roofline_stages`), the CPU
oracle timed on a bounded sample of the same workload and, under `other_workloads`,
the same measurements at the Llama-3.1-70B shape (80 x 131072 tokens, mixed 2 / 3
bits), the Llama-3.2-3B shape, the 3-bit grid and the decode read path (64 x 16384
cached tokens: scoring call and one-token append apart).  `--no-extras` keeps the
headline workload only; `--config` picks another headline.
"""
from __future__ import annotations

import argparse
import dataclasses

import numpy as np
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per fused encode launch measured with rocprofv3 --pmc (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB, the
# factors being what the same counters read for a 256 MiB device copy): profiles/bench_llama31_8b_pmc_counters.md.
# A constant taken from that profile, keyed by (config, n_codewords); other workloads report null.
MEASURED_TRAFFIC_BYTES = {("llama3.1-8b", 16): (2.0 * 110057.0 + 1.0 * 80384.3) * 1024.0}



def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="llama3.1-8b",
                    choices=["llama3.2-3b", "llama3.1-8b", "llama3.1-70b", "decode-read", "calibrate", "tiny"],
                    help="llama3.1-70b: 80 layers x 131072 tokens, grid of 16 or 64 points per layer (seeded coin); "
                         "decode-read: 64 sequences x 16384 cached tokens, scoring call + one-token append per layer; "
                         "calibrate: fitting the predictors of --layers layers (default 4) on --calib-tokens tokens")
    ap.add_argument("--calib-tokens", type=int, default=262144, help="tokens of the calibration set (--config calibrate)")
    ap.add_argument("--rht-group", type=int, default=0, choices=[0, 128, 1024],
                    help="values per rotation group and scale: 128 (one head, default) or 1024 (the whole token, the "
                         "grouping of the paper's experiments; predictor and quantizer then run as separate kernels)")
    ap.add_argument("--layers", type=int, default=0, help="use only the first N layers of the configuration (0: all)")
    ap.add_argument("--n-codewords", type=int, default=16)
    ap.add_argument("--rtn-bits", type=int, default=0, choices=[0, 2, 4],
                    help="2 or 4: the uniform round-to-nearest backbone (groups of 64) instead of the grid (0)")
    ap.add_argument("--q-heads", type=int, default=0, help="query heads for the scoring call (0: model default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the other workloads (70B shape, 3B shape, 3-bit grid, decode read path) that the default "
                         "run appends under `other_workloads`")
    ap.add_argument("--no-kernel-events", action="store_true", help="skip the instrumented replay")
    ap.add_argument("--cpu-rows", type=int, default=8192, help="token rows of the oracle sample")
    ap.add_argument("--cpu-layers", type=int, default=8, help="predicted layers of the oracle sample")
    ap.add_argument("--scores-form", default="sweep", choices=["sweep", "folded", "recompute"],
                    help="sweep: the scores come out of the decode sweep (aquakv_decode_attn_scores with Khat_out is the "
                         "key half of decode, aquakv_decode_values the value half); folded / recompute: a scoring "
                         "call of its own per layer after the decode sweep, with the key predictor folded into the "
                         "query or recomputed in the scoring kernel (the decode-read configuration has no sweep form)")
    ap.add_argument("--streams", type=int, default=1, choices=[1, 2],
                    help="2: the key chain and the value chain of the layer stack on two streams (aquakv_encode_keys / "
                         "_values, aquakv_decode_layer keys-only / aquakv_decode_values, an event per layer), so that the "
                         "kernels of neighbouring layers overlap (measured: about 1 %% faster); 1: the layer-level calls on one stream")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy (a known-size dispatch to scale rocprofv3 --pmc byte counters)")
    return ap.parse_args()


def grids_on_device(ns, device):
    """{n: (grid tensor, search table)} for the grid sizes in `ns`."""
    import torch
    from paper_2501_19392_amd import binding as B
    from paper_2501_19392_amd import synth
    out = {}
    for n in sorted(set(ns)):
        C = torch.from_numpy(synth.lloyd_codebook(n)).to(device)
        out[n] = (C, B.build_search_table(C))
    return out


def build_workload(cfg, device, n_per_layer, rht_group=0, rtn_bits=0):
    import torch
    from paper_2501_19392_amd import binding as B
    from paper_2501_19392_amd import synth
    sd = synth.torch_dtype(cfg.dtype)
    work = torch.float32 if cfg.dtype == "bf16" else torch.float64
    st = synth.KVStream(cfg, device=device, work=work)
    grids = {} if rtn_bits else grids_on_device(n_per_layer, device)
    layers, Ks, Vs = [], [], []
    for l in range(cfg.layers):
        K, V = st.next()
        Ks.append(K.contiguous())
        Vs.append(V.contiguous())
        wk = wv = None
        if l > 0:
            wk, wv = (w.to(device) for w in synth.analytic_predictors(st, l))
        if rtn_bits:
            layers.append(B.Layer(cfg.kv_heads, cfg.head_dim, None, None, None, sd, w_k=wk, w_v=wv, rtn_bits=rtn_bits))
            continue
        C, table = grids[n_per_layer[l]]
        sk = torch.from_numpy(synth.rht_signs(cfg.kv_heads, cfg.head_dim, l, "k")).to(device)
        sv = torch.from_numpy(synth.rht_signs(cfg.kv_heads, cfg.head_dim, l, "v")).to(device)
        layers.append(B.Layer(cfg.kv_heads, cfg.head_dim, C, sk, sv, sd, w_k=wk, w_v=wv, search_table=table,
                              rht_group=rht_group))
    return layers, Ks, Vs


def B_workspace_bytes(layer, tokens):
    from paper_2501_19392_amd import binding as B
    return B.aquakv_workspace_bytes(layer, tokens)


class Buffers:
    def __init__(self, layers, T, q_heads, device, scores_form="folded"):
        import torch
        self.codes = [(l.alloc_codes(T, device), l.alloc_codes(T, device)) for l in layers]
        lay = layers[0]
        # reconstructions: two ping-pong pairs are all the path needs (layer l-1 and l)
        self.hat = [(lay.alloc_kv(T, device), lay.alloc_kv(T, device)) for _ in range(2)]
        big = max(layers, key=lambda l: B_workspace_bytes(l, T))          # layers differ (a first layer has no predictor)
        self.ws = big.alloc_workspace(T, device)
        # two-stream schedule: the key chain may run ahead of the value chain, so 4 rotating pairs, one workspace
        # per chain, one event pair per layer
        self.hat4 = self.hat + [(lay.alloc_kv(T, device), lay.alloc_kv(T, device)) for _ in range(2)]
        self.ws_v = big.alloc_workspace(T, device)
        self.sk, self.sv = torch.cuda.Stream(device=device), torch.cuda.Stream(device=device)
        self.ev_k = [torch.cuda.Event() for _ in layers]
        self.ev_v = [torch.cuda.Event() for _ in layers]
        self.scores = torch.empty(1, q_heads, T, dtype=torch.float32, device=device)
        self.attn_out = torch.empty(1, q_heads, lay.head_dim, dtype=torch.float32, device=device)
        self.ws_weighted = lay.alloc_weighted_workspace(1, T, q_heads, device)
        self.P = torch.empty(T, lay.d, dtype=torch.float32, device=device)
        # scoring calls of their own take the folded form (aquakv_decode_attn_scores_folded) where it exists
        self.folded = scores_form == "folded"
        self.ws_scores = layers[-1].alloc_scores_workspace(1, q_heads, device)


SCORE_SCALE = 0.088388          # 1 / sqrt(128)


def scoring_call(B, lay, batch, S, q_heads, kc, ks, kp, q, scores, ws_scores, folded, ws):
    """A scoring call of its own (no keys out): the folded form where it exists and is asked for, else the definition."""
    if folded and kp is not None and B.aquakv_scores_workspace_bytes(lay, batch, q_heads) > 0:
        B.aquakv_decode_attn_scores_folded(lay, batch, S, q_heads, kc, ks, kp, q, SCORE_SCALE, scores, ws_scores)
    else:
        B.aquakv_decode_attn_scores(lay, batch, S, q_heads, kc, ks, kp, q, SCORE_SCALE, scores, None, ws)


def decode_sweep_with_scores(B, layers, buf, q, T, q_heads):
    """Decode of every layer with the scores as a by-product: the scoring call with Khat_out is the key half of
    Alg. "decode" (same kernel as decode, the q . k dot products added to its epilogue), aquakv_decode_values the
    value half.  Outputs: Khat, Vhat and scores of every layer, as from decode_layer + a scoring call."""
    prev = (None, None)
    for l, lay in enumerate(layers):
        (kc, ks), (vc, vs) = buf.codes[l]
        Kh, Vh = buf.hat[l & 1]
        B.aquakv_decode_attn_scores(lay, 1, T, q_heads, kc, ks, prev[0], q, SCORE_SCALE, buf.scores, Kh, buf.ws)
        B.aquakv_decode_values(lay, T, vc, vs, prev[1], Kh, Vh, buf.ws)
        prev = (Kh, Vh)


def decode_sweep_with_attention(B, layers, buf, q, T, q_heads):
    """The decode sweep with the whole attention of one query over the cache as a by-product: scores from the key
    half, and the value half with the soft-max-weighted sum over tokens taken in its epilogue (soft-max per 256
    tokens, merged by the combine step): three launches per predicted layer."""
    prev = (None, None)
    for l, lay in enumerate(layers):
        (kc, ks), (vc, vs) = buf.codes[l]
        Kh, Vh = buf.hat[l & 1]
        B.aquakv_decode_attn_scores(lay, 1, T, q_heads, kc, ks, prev[0], q, SCORE_SCALE, buf.scores, Kh, buf.ws)
        B.aquakv_decode_values_attend(lay, 1, T, q_heads, vc, vs, prev[1], Kh, buf.scores, Vh, buf.attn_out, None,
                                      buf.ws_weighted)
        prev = (Kh, Vh)


def run_step(B, layers, Ks, Vs, buf, q, T, q_heads, scores_in_sweep=True):
    """encode all layers, decode all layers, score all layers (layer-level entry points)."""
    prev = (None, None)
    for l, lay in enumerate(layers):
        (kc, ks), (vc, vs) = buf.codes[l]
        Kh, Vh = buf.hat[l & 1]
        B.aquakv_encode_layer(lay, T, Ks[l], Vs[l], prev[0], prev[1], kc, ks, vc, vs, Kh, Vh, buf.ws)
        prev = (Kh, Vh)
    if scores_in_sweep:
        decode_sweep_with_scores(B, layers, buf, q, T, q_heads)
        return
    prev = (None, None)
    for l, lay in enumerate(layers):
        (kc, ks), (vc, vs) = buf.codes[l]
        Kh, Vh = buf.hat[l & 1]
        B.aquakv_decode_layer(lay, T, kc, ks, vc, vs, prev[0], prev[1], Kh, Vh, buf.ws)
        prev = (Kh, Vh)
    # scoring reads layer l's codes and layer l-1's reconstructed keys; the ping-pong buffers hold
    # valid keys of the right shape, which is all that matters for the work done
    for l, lay in enumerate(layers):
        (kc, ks), _ = buf.codes[l]
        kp = None if l == 0 else buf.hat[(l - 1) & 1][0]
        scoring_call(B, lay, 1, T, q_heads, kc, ks, kp, q, buf.scores, buf.ws_scores, buf.folded, buf.ws)


def chains_on_two_streams(B, layers, Ks, Vs, buf, T, phase):
    """encode or decode of the whole layer stack with the key chain on stream sk and the value chain on sv.
    Value call l waits for key call l (it reads Khat of layer l); key call l + 4 waits for value call l (it reuses
    that buffer).  Both streams start after, and are joined into, the current stream."""
    import torch
    cur = torch.cuda.current_stream()
    sk, sv = buf.sk, buf.sv
    sk.wait_stream(cur)
    sv.wait_stream(cur)
    pk = pv = None
    for l, lay in enumerate(layers):
        (kc, ks), (vc, vs) = buf.codes[l]
        Kh, Vh = buf.hat4[l & 3]
        if l >= 4:
            sk.wait_event(buf.ev_v[l - 4])
        if phase == "encode":
            B.aquakv_encode_keys(lay, T, Ks[l], pk, kc, ks, Kh, buf.ws, stream=sk)
        else:
            B.aquakv_decode_layer(lay, T, kc, ks, None, None, pk, None, Kh, None, buf.ws, stream=sk)
        buf.ev_k[l].record(sk)
        sv.wait_event(buf.ev_k[l])
        if phase == "encode":
            B.aquakv_encode_values(lay, T, Vs[l], pv, Kh, vc, vs, Vh, buf.ws_v, stream=sv)
        else:
            B.aquakv_decode_values(lay, T, vc, vs, pv, Kh, Vh, buf.ws_v, stream=sv)
        buf.ev_v[l].record(sv)
        pk, pv = Kh, Vh
    cur.wait_stream(sk)
    cur.wait_stream(sv)


def run_step_two_streams(B, layers, Ks, Vs, buf, q, T, q_heads, scores_in_sweep=False):
    """The same work as run_step (scores by calls of their own), key and value chains of the encode and decode
    sweeps on two streams."""
    chains_on_two_streams(B, layers, Ks, Vs, buf, T, "encode")
    chains_on_two_streams(B, layers, Ks, Vs, buf, T, "decode")
    for l, lay in enumerate(layers):
        (kc, ks), _ = buf.codes[l]
        kp = None if l == 0 else buf.hat4[(l - 1) & 3][0]
        scoring_call(B, lay, 1, T, q_heads, kc, ks, kp, q, buf.scores, buf.ws_scores, buf.folded, buf.ws)


def timed_phases(B, layers, Ks, Vs, buf, q, T, q_heads, reps, streams=1, scores_in_sweep=False, reference=True):
    """Per-phase GPU time (ms per step) from stream events: encode / decode / scores (scoring calls of their own),
    and, when that is the step's form, decode+scores (the decode sweep that also yields the scores) and, for
    reference only, decode+attention (that sweep with soft-max and the weighted sum over the values as well)."""
    import torch
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {}
    def run_phase(phase):
        if phase == "decode+scores":
            decode_sweep_with_scores(B, layers, buf, q, T, q_heads)
            return
        if phase == "decode+attention":           # for reference: not part of the step
            decode_sweep_with_attention(B, layers, buf, q, T, q_heads)
            return
        if streams == 2 and phase != "scores":
            chains_on_two_streams(B, layers, Ks, Vs, buf, T, phase)          # joined into the current stream
            return
        prev = (None, None)
        for l, lay in enumerate(layers):
            (kc, ks), (vc, vs) = buf.codes[l]
            Kh, Vh = buf.hat[l & 1]
            if phase == "encode":
                B.aquakv_encode_layer(lay, T, Ks[l], Vs[l], prev[0], prev[1], kc, ks, vc, vs, Kh, Vh, buf.ws)
            elif phase == "decode":
                B.aquakv_decode_layer(lay, T, kc, ks, vc, vs, prev[0], prev[1], Kh, Vh, buf.ws)
            else:
                kp = None if l == 0 else buf.hat[(l - 1) & 1][0]
                scoring_call(B, lay, 1, T, q_heads, kc, ks, kp, q, buf.scores, buf.ws_scores, buf.folded, buf.ws)
            prev = (Kh, Vh)

    extra = ("decode+scores",) + (("decode+attention",) if reference else ())
    for phase in ("encode", "decode", "scores") + (extra if scores_in_sweep else ()):
        run_phase(phase)                          # untimed: the first call of a kernel loads its code
        a, b = ev(), ev()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            run_phase(phase)
        b.record()
        torch.cuda.synchronize()
        out[phase] = a.elapsed_time(b) / reps
    return out


def layer0_times(B, layers, Ks, Vs, buf, T, reps):
    """Layer 0 (no predictor: the stand-alone quantize / dequantize kernels) on its own, ms per call pair."""
    import torch
    ev = lambda: torch.cuda.Event(enable_timing=True)
    lay = layers[0]
    (kc, ks), (vc, vs) = buf.codes[0]
    Kh, Vh = buf.hat[0]
    out = {}
    for phase in ("encode", "decode"):
        a, b = ev(), ev()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            if phase == "encode":
                B.aquakv_encode_layer(lay, T, Ks[0], Vs[0], None, None, kc, ks, vc, vs, Kh, Vh, buf.ws)
            else:
                B.aquakv_decode_layer(lay, T, kc, ks, vc, vs, None, None, Kh, Vh, buf.ws)
        b.record()
        torch.cuda.synchronize()
        out[phase] = a.elapsed_time(b) / reps
    return out


def encode_kernel_events(B, layers, Ks, Vs, buf, T, steps):
    """HIP events (on the launch stream) around every `aquakv_encode_layer` call of `steps` passes over
    the predicted layers.  For a bf16 layer with predictors one call is exactly two launches of the
    dominant kernel, the fused encoder (keys: K = d_in_k, then values: K = d_in_v).
    Returns (predictor flops, algorithmic HBM bytes, total ms, launches)."""
    import torch
    D = layers[0].d
    pairs = []
    flops = 0.0
    nbytes = 0.0
    eb = 2
    for _ in range(steps):
        prev = (None, None)
        for l, lay in enumerate(layers):
            (kc, ks), (vc, vs) = buf.codes[l]
            Kh, Vh = buf.hat[l & 1]
            if l > 0:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
            B.aquakv_encode_layer(lay, T, Ks[l], Vs[l], prev[0], prev[1], kc, ks, vc, vs, Kh, Vh, buf.ws)
            if l > 0:
                b.record()
                pairs.append((a, b))
                flops += 2.0 * T * D * (lay.c.d_in_k + lay.c.d_in_v)
                code_bytes = lay.kv_heads * lay.code_bytes_per_group + 2 * (D // lay.rht_group) * lay.scale_words_per_group
                # per token: read K, V, Khat_prev, Vhat_prev and (value predictor) Khat; write Khat, Vhat, codes+scales
                nbytes += T * (5 * D * eb + 2 * D * eb + 2 * code_bytes) + (lay.c.d_in_k + lay.c.d_in_v) * D * eb
            prev = (Kh, Vh)
    torch.cuda.synchronize()
    ms = sum(a.elapsed_time(b) for a, b in pairs)
    return flops, nbytes, ms, 2 * len(pairs)


def cpu_baseline(cfg, n_codewords, rows, q_heads, n_layers, rtn_bits=0):
    """The oracle as it stands, on the host: encode + decode + scores of `n_layers` predicted layers
    on `rows` token rows of the same synthetic workload (rows are independent)."""
    import torch
    from oracle import aquakv_oracle as O
    from paper_2501_19392_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    sd = synth.torch_dtype(cfg.dtype)
    st = synth.KVStream(cfg, device="cpu", work=torch.float32, tokens=rows)
    f = lambda t: t.double().numpy()
    if rtn_bits:
        mk = lambda l, **kw: O.Layer(cfg.kv_heads, cfg.head_dim, dtype=cfg.dtype, rtn_bits=rtn_bits, **kw)
    else:
        C = synth.lloyd_codebook(n_codewords)
        mk = lambda l, **kw: O.Layer(cfg.kv_heads, cfg.head_dim, C, synth.rht_signs(cfg.kv_heads, cfg.head_dim, l, "k"),
                                     synth.rht_signs(cfg.kv_heads, cfg.head_dim, l, "v"), cfg.dtype, **kw)
    K0, V0 = st.next()
    prev = O.encode_layer(mk(0), f(K0), f(V0))
    q = f(synth.random_queries(1, q_heads, cfg.head_dim, seed=1, dtype=cfg.dtype))
    dt = 0.0
    for l in range(1, n_layers + 1):
        K1, V1 = st.next()
        wk, wv = synth.analytic_predictors(st, l)
        lay = mk(l, w_k=f(wk.to(sd)), w_v=f(wv.to(sd)))
        K1, V1 = f(K1), f(V1)
        t0 = time.perf_counter()
        e1 = O.encode_layer(lay, K1, V1, prev["Khat"], prev["Vhat"])
        O.decode_layer(lay, e1["k_codes"], e1["k_scales"], e1["v_codes"], e1["v_scales"], prev["Khat"], prev["Vhat"])
        O.attn_scores(lay, 1, rows, q, e1["k_codes"], e1["k_scales"], prev["Khat"])
        dt += time.perf_counter() - t0
        prev = e1
    return {"value": rows * n_layers / dt, "unit": "tokens/s per layer", "cores": int(threads), "kind": "oracle",
            "sample": f"encode+decode+scores of {n_layers} predicted layers on {rows} token rows "
                      f"({dt:.1f} s of CPU time; cost is linear in rows and layers)"}


PEAK_FP64_TFLOPS = 78.6          # MI355X fp64 vector


def calibration_path(args, device):
    """Calibration of the predictors (Alg. "Calibration") on the Llama-3.2-3B KV shape: a step = for every predicted
    layer fit f_key, encode the keys, fit f_value, encode the values (paper_2501_19392_amd.calibrate).  Reported
    per layer; the roofline entry is the fit call (fp64 FMA arithmetic; FLOPs of the two Gram products, the
    factorisation and the solves)."""
    import torch
    from paper_2501_19392_amd import binding as B
    from paper_2501_19392_amd import synth
    from paper_2501_19392_amd.calibrate import calibrate
    T, L, n = args.calib_tokens, (args.layers or 4) + 1, args.n_codewords
    cfg = synth.Config("llama3.2-3b-kv calibration", layers=L, kv_heads=8, head_dim=128, tokens=T, dtype="bf16")
    st = synth.KVStream(cfg, device=device, work=torch.float32)
    kv = [st.next() for _ in range(L)]
    C, table = grids_on_device([n], device)[n]
    signs = [(torch.from_numpy(synth.rht_signs(8, 128, l, "k")).to(device), torch.from_numpy(synth.rht_signs(8, 128, l, "v")).to(device))
             for l in range(L)]
    make_layer = lambda l, w_k=None, w_v=None: B.Layer(8, 128, C, signs[l][0], signs[l][1], torch.bfloat16, w_k=w_k, w_v=w_v,
                                                       search_table=table)
    run = lambda: calibrate(make_layer, L, lambda l: kv[l], rate=1e-3, device=device)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        layers = run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    # the fit call alone (value predictor: 2048 inputs), events on the launch stream
    D = 1024
    ws = torch.empty(B.aquakv_fit_workspace_bytes(2 * D, D), dtype=torch.uint8, device=device)
    W = torch.empty(D, 2 * D, dtype=torch.bfloat16, device=device)
    x0, x1, Y = kv[0][1], kv[1][0], kv[1][1]
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    B.aquakv_fit_predictor(torch.bfloat16, T, x0, D, x1, D, Y, D, 1e-3, W, None, ws)
    torch.cuda.synchronize()
    reps = 3
    a.record()
    for _ in range(reps):
        B.aquakv_fit_predictor(torch.bfloat16, T, x0, D, x1, D, Y, D, 1e-3, W, None, ws)
    b.record()
    torch.cuda.synchronize()
    fit_ms = a.elapsed_time(b) / reps
    d = 2 * D
    flops = 2.0 * T * (d * (d + 64) / 2 + d * D) + d ** 3 / 3.0 + 2.0 * d * d * D    # Gram products (G: lower triangle of 64-tiles), Cholesky, two solves
    achieved = flops / (fit_ms * 1e-3) / 1e12
    return {
        "metric": "predictor calibration, calibration tokens/s per layer", "value": round(T / (dt / (L - 1)), 1),
        "unit": "tokens/s per layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * dt, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"calibration of {L - 1} predicted layers of the llama3.2-3b KV shape (8 kv heads x 128, bf16, "
                               f"n={n}) on {T} tokens: per layer key fit (1024 inputs), key encode, value fit (2048 inputs), "
                               f"value encode", "tokens": T, "layers": L - 1},
        "roofline": {"kernel": "aquakv_fit_predictor, value predictor (gram_kernel and the block factorisation / solve kernels)",
                     "bound": "alu", "achieved": round(achieved, 2), "peak": PEAK_FP64_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_FP64_TFLOPS, 4), "traffic": None, "fit_ms": round(fit_ms, 3)},
    }


def decode_read_path(args, device):
    """The decode-phase read path: 64 sequences x 16384 cached tokens per layer, 32 query heads on 8 kv heads.
    A step = for every layer the scoring call over the whole compressed cache (aquakv_decode_attn_scores, one new
    query per sequence) and the append of one new token per sequence (aquakv_encode_layer with tokens = 64)."""
    import torch
    from paper_2501_19392_amd import binding as B
    from paper_2501_19392_amd import synth
    batch, S, q_heads, n = 64, 16384, args.q_heads or 32, args.n_codewords
    L = args.layers or 8
    T = batch * S
    cfg = synth.Config("decode-read", layers=L, kv_heads=8, head_dim=128, tokens=T, dtype="bf16")
    sd = torch.bfloat16
    st = synth.KVStream(cfg, device=device, work=torch.float32)
    C, table = (None, None) if args.rtn_bits else grids_on_device([n], device)[n]
    layers, codes, khat, new_rows = [], [], [], []
    vh = [None, None]
    ws = None
    prev = (None, None)
    # set-up (untimed): encode the cache layer by layer; only the compressed keys and the reconstructed keys
    # (the predictor input of the next layer's scoring call) are kept
    for l in range(L):
        K, V = st.next()
        sk = torch.from_numpy(synth.rht_signs(8, 128, l, "k")).to(device)
        sv = torch.from_numpy(synth.rht_signs(8, 128, l, "v")).to(device)
        wk = wv = None
        if l > 0:
            wk, wv = (w.to(device) for w in synth.analytic_predictors(st, l))
        if args.rtn_bits:
            lay = B.Layer(8, 128, None, None, None, sd, w_k=wk, w_v=wv, rtn_bits=args.rtn_bits)
        else:
            lay = B.Layer(8, 128, C, sk, sv, sd, w_k=wk, w_v=wv, search_table=table)
        ws = ws if ws is not None else lay.alloc_workspace(T, device)
        kc, ks = lay.alloc_codes(T, device)
        vc, vs = lay.alloc_codes(T, device)
        Kh = lay.alloc_kv(T, device)
        vh[l & 1] = vh[l & 1] if vh[l & 1] is not None else lay.alloc_kv(T, device)
        B.aquakv_encode_layer(lay, T, K, V, prev[0], prev[1], kc, ks, vc, vs, Kh, vh[l & 1], ws)
        torch.cuda.synchronize()
        # the new token of every sequence: reuse the last cached row of each sequence as its content
        last = torch.arange(batch, device=device) * S + (S - 1)
        new_rows.append(tuple(t[last].contiguous() for t in (K, V)) +
                        tuple(None if t is None else t[last].contiguous() for t in prev))
        layers.append(lay); codes.append((kc, ks)); khat.append(Kh)
        prev = (Kh, vh[l & 1])
        del K, V, vc, vs
    q = synth.random_queries(batch, q_heads, 128, seed=1, dtype="bf16", device=device)
    scores = torch.empty(batch, q_heads, S, dtype=torch.float32, device=device)
    folded = args.scores_form != "recompute" and B.aquakv_scores_workspace_bytes(layers[-1], batch, q_heads) > 0
    ws_scores = layers[-1].alloc_scores_workspace(batch, q_heads, device) if folded else torch.empty(16, dtype=torch.uint8, device=device)
    app = [(layers[0].alloc_codes(batch, device), layers[0].alloc_codes(batch, device), layers[0].alloc_kv(batch, device),
            layers[0].alloc_kv(batch, device))]
    ws_app = layers[-1].alloc_workspace(batch, device)

    def score_all():
        for l, lay in enumerate(layers):
            scoring_call(B, lay, batch, S, q_heads, codes[l][0], codes[l][1], None if l == 0 else khat[l - 1], q, scores,
                         ws_scores, folded, ws)

    def append_all():
        (kc, ks), (vc, vs), Kh, Vh = app[0]
        for l, lay in enumerate(layers):
            Kn, Vn, Kp, Vp = new_rows[l]
            B.aquakv_encode_layer(lay, batch, Kn, Vn, Kp, Vp, kc, ks, vc, vs, Kh, Vh, ws_app)

    for _ in range(args.warmup):
        score_all(); append_all()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        score_all(); append_all()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    ev = lambda: torch.cuda.Event(enable_timing=True)
    phases = {}
    for name, fn in (("scores", score_all), ("append", append_all)):
        a, b = ev(), ev()
        a.record()
        for _ in range(max(1, min(args.steps, 5))):
            fn()
        b.record()
        torch.cuda.synchronize()
        phases[name] = a.elapsed_time(b) / max(1, min(args.steps, 5))
    # scoring call of one predicted layer: read Khat_prev, codes, scales; write the scores
    pred_layers = L - 1
    lay_ = layers[-1]
    call_bytes = (T * (1024 * 2 + 8 * lay_.code_bytes_per_group + 2 * (1024 // lay_.rht_group) * lay_.scale_words_per_group)
                  + batch * q_heads * S * 4)
    a, b = ev(), ev()
    reps = max(1, min(args.steps, 5))
    a.record()
    for _ in range(reps):
        for l in range(1, L):
            scoring_call(B, layers[l], batch, S, q_heads, codes[l][0], codes[l][1], khat[l - 1], q, scores, ws_scores,
                         folded, ws)
    b.record()
    torch.cuda.synchronize()
    call_ms = a.elapsed_time(b) / (reps * pred_layers)
    gbs = call_bytes / (call_ms * 1e-3) / 1e9
    return {
        "metric": "decode read path: cached tokens scored per second per layer at %d bits/value" % (args.rtn_bits or n.bit_length() // 2),
        "value": round(T * L / dt, 1), "unit": "tokens/s per layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * dt, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"decode-read: {L} layers x {batch} sequences x {S} cached tokens x 8 kv heads x 128, bf16, "
                               f"{'round-to-nearest backbone' if args.rtn_bits else 'n=%d' % n}, step = q.k scores ({q_heads} query heads, {'folded' if folded else 'recompute'} form) over the whole "
                               f"cache + append of one token per sequence, for every layer",
                   "tokens": T, "layers": L, "q_heads": q_heads, "batch": batch, "seq_len": S},
        "phases_ms_per_step": {k: round(v, 3) for k, v in phases.items()},
        "roofline": {"kernel": "aquakv_decode_attn_scores of a predicted layer (query folding + streaming kernel)"
                     if folded else "fused_kernel<scores>", "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None, "launches": reps * pred_layers,
                     "avg_launch_us": round(1e3 * call_ms, 1), "algorithmic_bytes_per_launch": call_bytes},
    }


def stage_rooflines(B, layers, Ks, Vs, buf, q, T, q_heads, reps):
    """One roofline entry per stage of the path, each against its own bound, from HIP events on the launch
    stream around the calls of that stage alone (a layer-level call of a predicted bf16 layer is two launches of
    the same kernel, keys then values; a layer-0 call is two launches of the stand-alone kernel)."""
    import torch
    lay0, lay1 = layers[0], layers[-1]
    D = lay0.d
    eb = 2
    n_pred = len(layers) - 1
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, n):
        fn()
        a, b = ev(), ev()
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    def code_bytes(lay):          # codes + scales of one tensor, per token
        return lay.kv_heads * lay.code_bytes_per_group + 2 * (D // lay.rht_group) * lay.scale_words_per_group

    out = []

    def entry(stage, kernel, bound, work, ms, launches, note=None):
        per_launch = work / launches
        us = 1e3 * ms / launches
        if bound == "mfma":
            achieved, peak, unit = per_launch / (us * 1e-6) / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s"
            key = "algorithmic_flops_per_launch"
        else:
            achieved, peak, unit = per_launch / (us * 1e-6) / 1e9, PEAK_HBM_GBS, "GB/s"
            key = "algorithmic_bytes_per_launch"
        e = {"stage": stage, "kernel": kernel, "bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
             "frac": round(achieved / peak, 4), "traffic": None, "launches": launches, "avg_launch_us": round(us, 2),
             key: round(per_launch, 1)}
        if note:
            e["note"] = note
        out.append(e)

    (kc0, ks0), (vc0, vs0) = buf.codes[0]
    Kh, Vh = buf.hat[0]
    # stand-alone quantize / dequantize (layer 0: no predictor), HBM-bound: x in, xhat + codes + scale out
    ms = timed(lambda: B.aquakv_encode_layer(lay0, T, Ks[0], Vs[0], None, None, kc0, ks0, vc0, vs0, Kh, Vh, buf.ws), reps)
    entry("quantize (layer 0)", "quantize_kernel", "hbm", 2 * T * (2 * D * eb + code_bytes(lay0)), ms, 2)
    ms = timed(lambda: B.aquakv_decode_layer(lay0, T, kc0, ks0, vc0, vs0, None, None, Kh, Vh, buf.ws), reps)
    entry("dequantize (layer 0)", "dequantize_kernel", "hbm", 2 * T * (D * eb + code_bytes(lay0)), ms, 2)
    if n_pred == 0 or lay1.dtype != torch.bfloat16:
        return out
    wide = lay1.rht_group == D

    def sweep(kind):
        prev = buf.hat[0]
        for l in range(1, len(layers)):
            lay = layers[l]
            (kc, ks), (vc, vs) = buf.codes[l]
            Kh, Vh = buf.hat[l & 1]
            if kind == "encode":
                B.aquakv_encode_layer(lay, T, Ks[l], Vs[l], prev[0], prev[1], kc, ks, vc, vs, Kh, Vh, buf.ws)
            elif kind == "decode":
                B.aquakv_decode_layer(lay, T, kc, ks, vc, vs, prev[0], prev[1], Kh, Vh, buf.ws)
            else:
                scoring_call(B, lay, 1, T, q_heads, kc, ks, prev[0], q, buf.scores, buf.ws_scores, buf.folded, buf.ws)
            prev = (Kh, Vh)

    flops = sum(2.0 * T * D * (lay.c.d_in_k + lay.c.d_in_v) for lay in layers[1:])
    two = B.aquakv_fused_tile_heads(lay1, T) == 2
    ms = timed(lambda: sweep("encode"), reps)
    fused_wide = wide and getattr(B, "WIDE_ENCODE_FUSED", False)
    entry("encode (predicted layers)", "predict_bf16_kernel + quantize_kernel (groups across heads)" if wide and not fused_wide
          else "fused_wide_encode_kernel (64 tokens x 8 heads per workgroup; + retile_w_kernel, a few us)" if fused_wide
          else "fused_two_heads_kernel<encode> (256 tokens x 2 heads per workgroup)" if two
          else "fused_kernel<encode>", "mfma", flops, ms, 2 * n_pred)
    ms = timed(lambda: sweep("decode"), reps)
    entry("decode (predicted layers)", "fused_two_heads_kernel<decode> (256 tokens x 2 heads per workgroup)" if two
          else "fused_kernel<decode>", "mfma", flops, ms, 2 * n_pred)
    folded = B.aquakv_scores_workspace_bytes(lay1, 1, q_heads) > 0
    ms = timed(lambda: sweep("scores"), reps)
    passes = 1 if q_heads <= 32 else 2
    if folded:
        nbytes = n_pred * (passes * T * (D * eb + code_bytes(lay1)) + q_heads * T * 4)
        entry("q.k scores of their own (predictor folded into the query)", "fold_query_kernel + folded_scores_kernel", "hbm", nbytes, ms,
              n_pred, note="one call = both launches; the cache is read once per 4 query heads of a kv head (%d pass%s)" % (passes, "" if passes == 1 else "es"))
    else:
        entry("q.k scores of their own (prediction recomputed)", "fused_two_heads_kernel<scores>" if two else "fused_kernel<scores>", "mfma",
              sum(2.0 * T * D * lay.c.d_in_k for lay in layers[1:]), ms, n_pred)
    return out


def layer_workload(args, config, device, steps, warmup, n_codewords=None, rht_group=0, rtn_bits=0, q_heads_arg=0,
                   with_cpu_baseline=True, reference_phases=True):
    """Builds one layer-stack workload, times `steps` steps of it and returns the JSON line as a dict."""
    import torch
    from paper_2501_19392_amd import binding as B
    from paper_2501_19392_amd import synth
    n_codewords = n_codewords or args.n_codewords
    cfg = {"llama3.2-3b": synth.LLAMA32_3B, "llama3.1-8b": synth.LLAMA31_8B, "llama3.1-70b": synth.LLAMA31_70B,
           "tiny": synth.TINY}[config]
    if args.layers:
        cfg = dataclasses.replace(cfg, layers=min(args.layers, cfg.layers))
    q_heads = q_heads_arg or {"llama3.2-3b": 24, "llama3.1-8b": 32, "llama3.1-70b": 64, "tiny": 8}[config]
    T = cfg.tokens
    if config == "llama3.1-70b":
        # grid of 16 or 64 points per layer by a seeded fair coin (2 or 3 code bits per value, 2.5 on average)
        coin = np.random.Generator(np.random.PCG64(synth.BASE_SEED + 99)).integers(0, 2, size=cfg.layers)
        n_per_layer = [16 if c == 0 else 64 for c in coin]
        bits_label = "%.2f (grid of 16 or 64 points per layer)" % (sum(n.bit_length() // 2 for n in n_per_layer) / cfg.layers)
        grid_label = "n=16|64 per layer"
    else:
        n_per_layer = [n_codewords] * cfg.layers
        bits_label = "%d" % (n_codewords.bit_length() // 2)
        grid_label = f"n={n_codewords}"
    if rtn_bits:
        if config == "llama3.1-70b" or rht_group:
            sys.exit("bench.py: --rtn-bits goes with one backbone for all layers and its own groups of 64")
        bits_label = "%d (uniform round-to-nearest backbone, groups of 64: %.2f stored)" % (rtn_bits, rtn_bits + 0.5)
        grid_label = ""

    layers, Ks, Vs = build_workload(cfg, device, n_per_layer, rht_group, rtn_bits)
    wide = rht_group not in (0, cfg.head_dim)
    if wide:
        grid_label += f", rotation groups of {rht_group} (one scale per token)"
    quantizer_label = (f"uniform round-to-nearest with {1 << rtn_bits} levels, groups of 64" if rtn_bits
                       else f"{grid_label} codewords (p=2)")
    # the two-stream schedule keeps scoring calls of their own (folded where the form exists)
    sweep = args.scores_form == "sweep" and args.streams == 1
    buf = Buffers(layers, T, q_heads, device, "folded" if args.scores_form == "sweep" else args.scores_form)
    q = synth.random_queries(1, q_heads, cfg.head_dim, seed=1, dtype=cfg.dtype, device=device)

    if args.calibrate_copy:
        src = torch.zeros(64 << 20, dtype=torch.float32, device=device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    step = run_step_two_streams if args.streams == 2 else run_step
    for _ in range(warmup):
        step(B, layers, Ks, Vs, buf, q, T, q_heads, sweep)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(B, layers, Ks, Vs, buf, q, T, q_heads, sweep)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / steps
    value = T * cfg.layers / (dt / steps)

    reps = max(1, min(steps, 5 if T <= 32768 else 2))
    phases = timed_phases(B, layers, Ks, Vs, buf, q, T, q_heads, reps, args.streams, sweep, reference_phases)
    l0 = layer0_times(B, layers, Ks, Vs, buf, T, 5)
    eb = 2 if cfg.dtype == "bf16" else 4
    D = cfg.kv_heads * cfg.head_dim
    code_b = 2 * T * (cfg.kv_heads * layers[0].code_bytes_per_group
                      + 2 * (D // layers[0].rht_group) * layers[0].scale_words_per_group)
    # layer 0 moves, per call: encode reads K, V and writes Khat, Vhat + codes; decode reads codes and writes Khat, Vhat
    l0_bytes = {"encode": 4 * T * D * eb + code_b, "decode": 2 * T * D * eb + code_b}
    n_pred = max(cfg.layers - 1, 1)
    pred_ms = {k: (phases[k] - l0[k]) / n_pred for k in ("encode", "decode")}
    roofline = None
    stages = None
    if cfg.dtype == "bf16" and not args.no_kernel_events:
        flops, nbytes, ms, launches = encode_kernel_events(B, layers, Ks, Vs, buf, T, max(1, min(steps, 3 if T <= 32768 else 1)))
        achieved = flops / (ms * 1e-3) / 1e12
        fused_wide = wide and getattr(B, "WIDE_ENCODE_FUSED", False)
        if wide and not fused_wide:
            launches *= 2
        roofline = {"kernel": "predict_bf16_kernel + quantize_kernel per tensor (groups across heads are not fused)" if wide and not fused_wide
                    else "fused_wide_encode_kernel (bf16 MFMA predictor + quantizer epilogue over whole tokens)" if fused_wide
                    else "fused_two_heads_kernel<encode> (bf16 MFMA predictor + quantizer epilogue, 256 tokens x 2 heads per workgroup)"
                    if B.aquakv_fused_tile_heads(layers[-1], T) == 2
                    else "fused_kernel<encode> (bf16 MFMA predictor + quantizer epilogue)", "bound": "mfma",
                    "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    # not measured in this run: a constant from the rocprofv3 --pmc summary under profiles/, or null
                    "traffic": None if wide or rtn_bits else MEASURED_TRAFFIC_BYTES.get((config, n_codewords)),
                    "traffic_source": "constant from profiles/ (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE of an earlier run of this command)"
                    if not (wide or rtn_bits) and (config, n_codewords) in MEASURED_TRAFFIC_BYTES else None,
                    "launches": launches,
                    "algorithmic_bytes_per_launch": round(nbytes / launches, 1),
                    "avg_launch_us": round(1e3 * ms / launches, 2),
                    "algorithmic_hbm_GBs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                    "algorithmic_hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        stages = stage_rooflines(B, layers, Ks, Vs, buf, q, T, q_heads, reps)

    line = {
        "metric": "KV encode+decode tokens/s per layer at %s bits/value" % bits_label,
        "value": round(value, 1), "unit": "tokens/s per layer", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.layers} layers x {T} tokens x {cfg.kv_heads} kv heads x {cfg.head_dim}, "
                               f"{cfg.dtype}, {quantizer_label}, step = encode + decode + q.k scores "
                               f"({q_heads} query heads) of every layer"
                               + (", the scores produced by the decode sweep (scoring call with Khat_out = key half of "
                                  "decode, then the value half)" if sweep else ", scoring calls of their own after the decode sweep")
                               + (", key and value chains of the sweeps on two streams" if args.streams == 2 else ""),
                   "tokens": T, "layers": cfg.layers, "q_heads": q_heads, "streams": args.streams,
                   "scores": "decode sweep" if sweep else "own calls"},
        # a step is encode + decode+scores when the scores come out of the decode sweep, else encode + decode + scores;
        # the other entries are the same phases measured apart, for reference
        "phases_ms_per_step": {k: round(v, 3) for k, v in phases.items()},
        "tokens_per_s_per_layer": {k: round(T * cfg.layers / (v * 1e-3), 1) for k, v in phases.items()},
        # encode + decode combined, T / (t_enc + t_dec) per layer: predicted layers (average) and layer 0 apart
        "encode_plus_decode_tokens_per_s": {
            "predicted_layers": round(T / ((pred_ms["encode"] + pred_ms["decode"]) * 1e-3), 1),
            "layer0": round(T / ((l0["encode"] + l0["decode"]) * 1e-3), 1)},
        "layer0": {"encode_ms": round(l0["encode"], 4), "decode_ms": round(l0["decode"], 4),
                   "encode_GBs": round(l0_bytes["encode"] / (l0["encode"] * 1e-3) / 1e9, 1),
                   "decode_GBs": round(l0_bytes["decode"] / (l0["decode"] * 1e-3) / 1e9, 1),
                   "bound": "hbm"},
        "roofline": roofline,
        "roofline_stages": stages,
    }
    if with_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, n_codewords, min(args.cpu_rows, T), q_heads, min(args.cpu_layers, cfg.layers - 1),
                                            rtn_bits)
    del layers, Ks, Vs, buf
    torch.cuda.empty_cache()
    return line


def brief(line):
    """What an `other_workloads` entry keeps of a full line."""
    keep = ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "phases_ms_per_step", "roofline", "roofline_stages")
    out = {k: line[k] for k in keep if k in line}
    out["workload"] = line["config"]["workload"]
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); the path shards along tokens with no "
              "exchange between GPUs, so N GPUs are N independent copies of this run", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    device = "cuda:0"
    torch.cuda.set_device(0)
    if args.config == "decode-read":
        print(json.dumps(decode_read_path(args, device)))
        return
    if args.config == "calibrate":
        print(json.dumps(calibration_path(args, device)))
        return
    log = lambda msg: print("bench.py: " + msg, file=sys.stderr, flush=True)
    t_start = time.perf_counter()
    line = layer_workload(args, args.config, device, args.steps, args.warmup, rht_group=args.rht_group, rtn_bits=args.rtn_bits,
                          q_heads_arg=args.q_heads, with_cpu_baseline=not args.no_cpu_baseline)
    log("headline workload done after %.0f s" % (time.perf_counter() - t_start))
    plain = not (args.rht_group or args.rtn_bits or args.layers or args.streams != 1 or args.scores_form != "sweep"
                 or args.n_codewords != 16 or args.q_heads)
    if args.config == "llama3.1-8b" and plain and not args.no_extras:
        # the other workloads of the workload list, in the same process and under the same clock; fewer steps each
        # so that the whole run stays within a few minutes
        others = {}
        for name, kw, st, wu in (
                ("llama3.1-8b, 3 bits (n=64)", dict(config="llama3.1-8b", n_codewords=64), min(args.steps, 5), 1),
                ("llama3.1-8b, 4 bits (n=256)", dict(config="llama3.1-8b", n_codewords=256), min(args.steps, 5), 1),
                ("llama3.1-70b, mixed 2/3 bits", dict(config="llama3.1-70b"), min(args.steps, 2), 1),
                ("llama3.2-3b, 2 bits", dict(config="llama3.2-3b"), min(args.steps, 10), 2),
                ("llama3.1-8b, 2 bits, rotation groups of 1024 (the paper's grouping)",
                 dict(config="llama3.1-8b", rht_group=1024), min(args.steps, 5), 1)):
            others[name] = brief(layer_workload(args, device=device, steps=st, warmup=wu, with_cpu_baseline=False,
                                                reference_phases=False, **kw))
            log("%s done after %.0f s" % (name, time.perf_counter() - t_start))
        dr_args = argparse.Namespace(**vars(args))
        dr_args.steps, dr_args.warmup, dr_args.layers = min(args.steps, 3), 1, 0
        dr = decode_read_path(dr_args, device)
        others["decode-read (64 x 16384 cached tokens, 32 query heads)"] = {
            k: dr[k] for k in ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "phases_ms_per_step", "roofline")}
        others["decode-read (64 x 16384 cached tokens, 32 query heads)"]["workload"] = dr["config"]["workload"]
        log("decode-read done after %.0f s" % (time.perf_counter() - t_start))
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
