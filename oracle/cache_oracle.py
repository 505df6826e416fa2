"""CPU oracle of the cache policy around the per-layer encode / decode calls.

TEST INFRASTRUCTURE ONLY (same rules as aquakv_oracle.py: imported by tests only, shares no
code with the product package).

What it follows (AQUA-KV paper, arxiv 2501.19392):
  * Sect. 3.3 "Relation between AQUA-KV and Attention Sinks": the first few tokens (4 in the
    experiments) stay uncompressed.
  * Sect. 3.3 "Inference Algorithm" and Alg. "Inference": a buffer of up to r = 128 recent tokens
    is kept uncompressed; when it is full its contents are quantized layer by layer from the first
    layer to the last (each layer's predictors read the previous layer's reconstruction of the same
    tokens); to attend, the past is recovered one layer at a time with Alg. "decode", every layer
    from the previous layer's recovered past.

  * Sect. 4.1 (first-layer strategies, Table 1 "1st Layer Keys & Values"): the first layer has no predictor and
    is either quantized by the backbone alone (the default for the Llama models: a 4-bit grid) or kept in 16
    bits (the Qwen setting).  Here every layer brings its own grid, and a layer given as None is kept in 16 bits:
    its flushed tokens are stored as they are and feed the next layer's predictors exactly.

Quantization is per token, so flushing the buffer in pieces gives the same codes as encoding the
same token range in one call; the pin in tests/test_cache_policy.py checks exactly that, and that
sinks and buffered tokens come back untouched.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import aquakv_oracle as O


class CacheOracle:
    def __init__(self, layers: Sequence[O.Layer], sink_tokens: int = 4, buffer_tokens: int = 128):
        self.layers = list(layers)
        self.sink_tokens, self.buffer_tokens = sink_tokens, buffer_tokens
        L = len(self.layers)
        empty = lambda: [None] * L
        self.sink_k, self.sink_v = empty(), empty()          # [<= sink_tokens, H, g] as given
        self.buf_k, self.buf_v = empty(), empty()            # [<  buffer_tokens, H, g] as given
        self.codes = [dict(k_codes=[], k_scales=[], v_codes=[], v_scales=[]) for _ in range(L)]
        self.raw = [dict(k=[], v=[]) for _ in range(L)]      # flushed tokens of the layers kept in 16 bits
        self.n_sink = self.n_compressed = self.n_buffered = 0

    @property
    def n_tokens(self):
        return self.n_sink + self.n_compressed + self.n_buffered

    @staticmethod
    def _cat(a, b):
        return b if a is None else np.concatenate([a, b], axis=0)

    def append(self, kv: Sequence[Tuple[np.ndarray, np.ndarray]]):
        """kv[l] = (K, V) of the new tokens at layer l, [t, H, g] holding storage-dtype values."""
        t = kv[0][0].shape[0]
        pos = 0
        while pos < t:
            if self.n_sink < self.sink_tokens:
                take = min(self.sink_tokens - self.n_sink, t - pos)
                for l, (K, V) in enumerate(kv):
                    self.sink_k[l] = self._cat(self.sink_k[l], np.asarray(K[pos:pos + take], dtype=np.float64))
                    self.sink_v[l] = self._cat(self.sink_v[l], np.asarray(V[pos:pos + take], dtype=np.float64))
                self.n_sink += take
            else:
                take = min(self.buffer_tokens - self.n_buffered, t - pos)
                for l, (K, V) in enumerate(kv):
                    self.buf_k[l] = self._cat(self.buf_k[l], np.asarray(K[pos:pos + take], dtype=np.float64))
                    self.buf_v[l] = self._cat(self.buf_v[l], np.asarray(V[pos:pos + take], dtype=np.float64))
                self.n_buffered += take
                if self.n_buffered == self.buffer_tokens:
                    self._flush()
            pos += take

    def _flush(self):
        """The full buffer is quantized from the first layer to the last (Alg. "encode" per layer)."""
        Kp = Vp = None
        for l, lay in enumerate(self.layers):
            if lay is None:                                   # kept in 16 bits: stored as is
                self.raw[l]["k"].append(self.buf_k[l]); self.raw[l]["v"].append(self.buf_v[l])
                Kp, Vp = self.buf_k[l], self.buf_v[l]
            else:
                e = O.encode_layer(lay, self.buf_k[l], self.buf_v[l], Kp, Vp)
                for name in ("k_codes", "k_scales", "v_codes", "v_scales"):
                    self.codes[l][name].append(e[name])
                Kp, Vp = e["Khat"], e["Vhat"]
            self.buf_k[l] = self.buf_v[l] = None
        self.n_compressed += self.n_buffered
        self.n_buffered = 0

    def sweep(self):
        """Yield (layer, K, V) for every layer in order: sinks, recovered compressed past, buffered tokens.
        Only one layer's past is alive at a time (Alg. "Inference", first line of the loop)."""
        Kp = Vp = None
        for l, lay in enumerate(self.layers):
            parts_k, parts_v = [], []
            if self.n_sink:
                parts_k.append(self.sink_k[l]); parts_v.append(self.sink_v[l])
            if self.n_compressed:
                if lay is None:
                    Kp, Vp = np.concatenate(self.raw[l]["k"], axis=0), np.concatenate(self.raw[l]["v"], axis=0)
                else:
                    c = {k: np.concatenate(v, axis=0) for k, v in self.codes[l].items()}
                    Kp, Vp = O.decode_layer(lay, c["k_codes"], c["k_scales"], c["v_codes"], c["v_scales"], Kp, Vp)
                parts_k.append(Kp); parts_v.append(Vp)
            if self.n_buffered:
                parts_k.append(self.buf_k[l]); parts_v.append(self.buf_v[l])
            yield l, np.concatenate(parts_k, axis=0), np.concatenate(parts_v, axis=0)

    def attend(self, queries, score_scale: float, rope=None):
        """Attention of one new token's queries over everything cached (Alg. "Inference", the block call with
        K = [recovered past], one token): queries[l] is [q_heads, head_dim]; returns one [q_heads, head_dim] per layer.
        The soft-max runs over sinks, recovered compressed tokens and buffered tokens alike.  rope = (cos, sin), each
        [>= n_tokens, head_dim/2]: the cache holds keys from before the rotary embedding; token t is rotated by row t."""
        out = []
        n = self.n_tokens
        for l, K, V in self.sweep():
            o, _, _ = O.attention(np.asarray(queries[l], dtype=np.float64)[None], K[None], V[None], score_scale,
                                  None if rope is None else (np.asarray(rope[0])[:n], np.asarray(rope[1])[:n]))
            out.append(o[0])
        return out

    def stored_bytes(self, elem_bytes: int = 2) -> int:
        """Bytes held for all layers: uncompressed sinks and buffer, packed codes and fp16 scales."""
        some = next(l for l in self.layers if l is not None)
        per_tok = some.kv_heads * some.head_dim * elem_bytes * 2
        raw = (self.n_sink + self.n_buffered) * per_tok * len(self.layers)
        raw += sum(int(a.size) * elem_bytes for r in self.raw for v in r.values() for a in v)
        comp = sum(int(a.size) * a.itemsize for c in self.codes for v in c.values() for a in v)
        return raw + comp
