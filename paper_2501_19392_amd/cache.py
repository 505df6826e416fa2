"""Cache policy around the per-layer calls: attention sinks, recent-token buffer, flush and recovery.

AQUA-KV paper (arxiv 2501.19392), Sect. 3.3: the first few tokens ("attention sinks", 4 in the
experiments) stay in 16 bits; up to r = 128 recent tokens are kept uncompressed and, when that buffer
is full, quantized layer by layer from the first layer to the last; Alg. "Inference": to attend, the
compressed past is recovered one layer at a time, each layer from the previous layer's recovered past.

Sect. 4.1 (first-layer strategies): every layer brings its own grid (the paper's default quantizes the first layer,
which has no predictor, with the 4-bit grid), and a layer given as None is kept in 16 bits (its flushed tokens are
stored as they are and feed the next layer's predictors).

`attend` is the block call of Alg. "Inference" for one new token as far as the cache is concerned: per layer the
soft-max attention of that token's queries over everything cached.  The compressed range is scored and summed by the
decode kernels themselves (`aquakv_decode_attn_scores` with the keys as output, `aquakv_decode_values_attend`), the
sinks and the buffer by `aquakv_attend_raw`, which merges its share into the running result.

This class is bookkeeping only: every number is produced by the C-ABI calls (`aquakv_encode_layer`,
`aquakv_decode_layer`, the attention calls above); torch tensors are the device memory they work on.  One sequence per
cache.
"""
from __future__ import annotations

from typing import Iterator, List, Sequence, Tuple

import torch

from . import binding as B


class AquaKVCache:
    def __init__(self, layers: Sequence[B.Layer], max_tokens: int, sink_tokens: int = 4, buffer_tokens: int = 128,
                 device="cuda"):
        if buffer_tokens < 1 or sink_tokens < 0:
            raise ValueError("buffer_tokens >= 1 and sink_tokens >= 0")
        self.layers = list(layers)
        self.sink_tokens, self.buffer_tokens, self.max_tokens = sink_tokens, buffer_tokens, max_tokens
        lay0 = next(l for l in self.layers if l is not None)
        H, g, dt = lay0.kv_heads, lay0.head_dim, lay0.dtype
        raw = lambda t: torch.empty(t, H, g, dtype=dt, device=device)
        self.sink = [(raw(max(sink_tokens, 1)), raw(max(sink_tokens, 1))) for _ in self.layers]
        self.buf = [(raw(buffer_tokens), raw(buffer_tokens)) for _ in self.layers]
        cap = max(max_tokens - sink_tokens, 0) // buffer_tokens * buffer_tokens      # the compressed range grows by whole buffers
        self.codes = [None if l is None else (l.alloc_codes(max(cap, 1), device), l.alloc_codes(max(cap, 1), device))
                      for l in self.layers]
        self.raw = [(raw(max(cap, 1)), raw(max(cap, 1))) if l is None else None for l in self.layers]   # layers kept in 16 bits
        self.capacity = cap
        # flush: reconstructions of the flushed tokens, two ping-pong pairs (layer l - 1 feeds layer l)
        self._flush_hat = [(raw(buffer_tokens), raw(buffer_tokens)) for _ in range(2)]
        coded = [l for l in self.layers if l is not None]
        self._flush_ws = max((l.alloc_workspace(buffer_tokens, device) for l in coded), key=lambda t: t.numel())
        # recovery: [sinks | compressed | buffer] of one layer, two ping-pong pairs
        self._view = [(raw(max_tokens), raw(max_tokens)) for _ in range(2)]
        self._view_ws = max((l.alloc_workspace(max(cap, 1), device) for l in coded), key=lambda t: t.numel())
        self.n_sink = self.n_compressed = self.n_buffered = 0
        self._attend = None                 # buffers of attend(), sized on first use (they depend on the query heads)
        self._device = device

    @property
    def n_tokens(self) -> int:
        return self.n_sink + self.n_compressed + self.n_buffered

    def append(self, kv: Sequence[Tuple[torch.Tensor, torch.Tensor]]) -> None:
        """kv[l] = (K, V) of the new tokens at layer l, [t, kv_heads, head_dim] in the storage dtype."""
        if len(kv) != len(self.layers):
            raise ValueError("one (K, V) pair per layer")
        t = kv[0][0].shape[0]
        if self.n_tokens + t > self.max_tokens:
            raise ValueError("cache is full")
        pos = 0
        while pos < t:
            if self.n_sink < self.sink_tokens:
                take = min(self.sink_tokens - self.n_sink, t - pos)
                for l, (K, V) in enumerate(kv):
                    self.sink[l][0][self.n_sink:self.n_sink + take].copy_(K[pos:pos + take])
                    self.sink[l][1][self.n_sink:self.n_sink + take].copy_(V[pos:pos + take])
                self.n_sink += take
            else:
                take = min(self.buffer_tokens - self.n_buffered, t - pos)
                for l, (K, V) in enumerate(kv):
                    self.buf[l][0][self.n_buffered:self.n_buffered + take].copy_(K[pos:pos + take])
                    self.buf[l][1][self.n_buffered:self.n_buffered + take].copy_(V[pos:pos + take])
                self.n_buffered += take
                if self.n_buffered == self.buffer_tokens:
                    self._flush()
            pos += take

    def _flush(self) -> None:
        """The full buffer is quantized from the first layer to the last; codes land behind the compressed range."""
        r, at = self.buffer_tokens, self.n_compressed
        Kp = Vp = None
        for l, lay in enumerate(self.layers):
            if lay is None:                                  # kept in 16 bits: stored as is, feeds the next layer exactly
                Kp, Vp = self.raw[l][0][at:at + r], self.raw[l][1][at:at + r]
                Kp.copy_(self.buf[l][0]); Vp.copy_(self.buf[l][1])
                continue
            (kc, ks), (vc, vs) = self.codes[l]
            Kh, Vh = self._flush_hat[l & 1]
            B.aquakv_encode_layer(lay, r, self.buf[l][0], self.buf[l][1], Kp, Vp, kc[at:at + r], ks[at:at + r],
                                  vc[at:at + r], vs[at:at + r], Kh, Vh, self._flush_ws)
            Kp, Vp = Kh, Vh
        self.n_compressed += r
        self.n_buffered = 0

    def sweep(self) -> Iterator[Tuple[int, torch.Tensor, torch.Tensor]]:
        """Yield (layer, K, V) for every layer in order, K and V being [n_tokens, kv_heads, head_dim]: sinks, the
        recovered compressed past, the buffered tokens.  The tensors are views of two ping-pong buffers: layer l's
        are valid until layer l + 2 is produced."""
        s, c, b = self.n_sink, self.n_compressed, self.n_buffered
        Kp = Vp = None
        for l, lay in enumerate(self.layers):
            K, V = self._view[l & 1]
            if s:
                K[:s].copy_(self.sink[l][0][:s]); V[:s].copy_(self.sink[l][1][:s])
            if c and lay is None:
                K[s:s + c].copy_(self.raw[l][0][:c]); V[s:s + c].copy_(self.raw[l][1][:c])
                Kp, Vp = K[s:s + c], V[s:s + c]
            elif c:
                (kc, ks), (vc, vs) = self.codes[l]
                B.aquakv_decode_layer(lay, c, kc[:c], ks[:c], vc[:c], vs[:c], Kp, Vp, K[s:s + c], V[s:s + c], self._view_ws)
                Kp, Vp = K[s:s + c], V[s:s + c]
            if b:
                K[s + c:s + c + b].copy_(self.buf[l][0][:b]); V[s + c:s + c + b].copy_(self.buf[l][1][:b])
            yield l, K[:s + c + b], V[:s + c + b]

    def attend(self, queries: Sequence[torch.Tensor], score_scale: float, rope=None) -> List[torch.Tensor]:
        """queries[l]: [q_heads, head_dim] in the storage dtype, the new token's queries at layer l.  Returns one
        fp32 [q_heads, head_dim] per layer: softmax(score_scale * q K^T) V over sinks, compressed past and buffer.
        One sweep over the layers; the recovered tensors of layer l feed layer l + 1 as in `sweep`.
        rope = (cos, sin), device fp32 [>= n_tokens, head_dim / 2]: the cache holds keys from before the rotary
        embedding (Sect. 3.3, the paper's default); the key of token t is rotated by row t on the fly, the queries
        are taken as already rotated, and what is recovered for the next layer stays unrotated."""
        s, c, b = self.n_sink, self.n_compressed, self.n_buffered
        if s + c + b == 0:
            raise ValueError("nothing cached")
        lay0 = next(l for l in self.layers if l is not None)
        H, g, dt = lay0.kv_heads, lay0.head_dim, lay0.dtype
        QH = queries[0].shape[0]
        if self._attend is None or self._attend["q_heads"] != QH:
            cap = max(self.capacity, 1)
            coded = [l for l in self.layers if l is not None]
            self._attend = dict(
                q_heads=QH,
                scores=torch.empty(QH * cap, dtype=torch.float32, device=self._device),
                out=[torch.empty(1, QH, g, dtype=torch.float32, device=self._device) for _ in self.layers],
                stats=torch.empty(1, QH, 2, dtype=torch.float32, device=self._device),
                ws=max((l.alloc_weighted_workspace(1, cap, QH, self._device) for l in coded), key=lambda t: t.numel()))
        A = self._attend
        step = 4096                                              # tokens per aquakv_attend_raw call
        cos, sin = rope if rope is not None else (None, None)
        rows = lambda t, a, n: None if t is None else t[a:a + n]  # the angles of tokens a ... a + n - 1
        Kp = Vp = None
        for l, lay in enumerate(self.layers):
            q = queries[l].reshape(1, QH, g)
            out, stats = A["out"][l], A["stats"]
            have = False
            if c and lay is None:                                # compressed range kept in 16 bits
                Kp, Vp = self.raw[l][0][:c], self.raw[l][1][:c]
                for r0 in range(0, c, step):
                    n = min(step, c - r0)
                    B.aquakv_attend_raw(dt, 1, n, H, QH, Kp[r0:r0 + n], Vp[r0:r0 + n], q, score_scale, out, stats, have,
                                        rope_cos=rows(cos, s + r0, n), rope_sin=rows(sin, s + r0, n))
                    have = True
            elif c:
                (kc, ks), (vc, vs) = self.codes[l]
                K, V = self._view[l & 1]
                scores = A["scores"][:QH * c].view(1, QH, c)
                if rope is None:
                    B.aquakv_decode_attn_scores(lay, 1, c, QH, kc[:c], ks[:c], Kp, q, score_scale, scores, K[:c], self._view_ws)
                else:
                    B.aquakv_decode_attn_scores_rope(lay, 1, c, QH, kc[:c], ks[:c], Kp, q, rows(cos, s, c), rows(sin, s, c),
                                                     score_scale, scores, K[:c], self._view_ws)
                B.aquakv_decode_values_attend(lay, 1, c, QH, vc[:c], vs[:c], Vp, K[:c], scores, V[:c], out, stats, A["ws"])
                Kp, Vp = K[:c], V[:c]
                have = True
            if s:
                B.aquakv_attend_raw(dt, 1, s, H, QH, self.sink[l][0][:s], self.sink[l][1][:s], q, score_scale, out, stats, have,
                                    rope_cos=rows(cos, 0, s), rope_sin=rows(sin, 0, s))
                have = True
            for r0 in range(0, b, step):
                n = min(step, b - r0)
                B.aquakv_attend_raw(dt, 1, n, H, QH, self.buf[l][0][r0:r0 + n], self.buf[l][1][r0:r0 + n], q, score_scale,
                                    out, stats, have, rope_cos=rows(cos, s + c + r0, n), rope_sin=rows(sin, s + c + r0, n))
                have = True
        return [o[0] for o in A["out"]]

    def stored_bytes(self) -> int:
        """Bytes the cache content occupies (all layers): 16-bit sinks and buffer, packed codes and fp16 scales."""
        lay0 = next(l for l in self.layers if l is not None)
        per_tok = lay0.d * self.sink[0][0].element_size() * 2
        total = (self.n_sink + self.n_buffered) * per_tok * len(self.layers)
        for lay in self.layers:
            if lay is None:
                total += self.n_compressed * per_tok
                continue
            groups = lay.d // lay.rht_group
            total += 2 * self.n_compressed * (lay.kv_heads * lay.code_bytes_per_group + 2 * groups * lay.scale_words_per_group)
        return total
