"""Cache policy around the per-layer calls: attention sinks, recent-token buffer, flush and recovery, for a batch
of sequences.

AQUA-KV paper (arxiv 2501.19392), Sect. 3.3: the first few tokens ("attention sinks", 4 in the
experiments) stay in 16 bits; up to r = 128 recent tokens are kept uncompressed and, when that buffer
is full, quantized layer by layer from the first layer to the last; Alg. "Inference": to attend, the
compressed past is recovered one layer at a time, each layer from the previous layer's recovered past.

Sect. 4.1 (first-layer strategies): every layer brings its own grid (the paper's default quantizes the first layer,
which has no predictor, with the 4-bit grid), and a layer given as None is kept in 16 bits (its flushed tokens are
stored as they are and feed the next layer's predictors).

`attend` is the block call of Alg. "Inference" for one new token per sequence as far as the cache is concerned: per
layer the soft-max attention of that token's queries over everything cached.  The compressed range is scored and
summed by the decode kernels themselves (`aquakv_decode_attn_scores` with the keys as output,
`aquakv_decode_values_attend`), the sinks and the buffer by `aquakv_attend_raw`, which merges its share into the
running result.

Batch.  Every sequence has its own sinks, buffer and compressed range (lengths may differ).  All sequences whose
buffer fills during one `append` are quantized together: ONE `aquakv_encode_layer` per layer over
(number of full buffers) x r tokens.  `attend` treats the sequences that hold the same number of compressed tokens as
one batch of the decode calls (`batch` x `seq_len` is what those calls take); in lock-step decoding from prompts of
one length that is the whole batch.  Codes of a sequence are contiguous in its own range of the code tensors, so a
group of several sequences is first gathered into one token-major staging range (codes are an eighth of the bytes the
decode call moves).

This class is bookkeeping only: every number is produced by the C-ABI calls (`aquakv_encode_layer`,
`aquakv_decode_layer`, the attention calls above); torch tensors are the device memory they work on.
"""
from __future__ import annotations

from typing import Dict, Iterator, List, Optional, Sequence, Tuple

import torch

from . import binding as B


class AquaKVCache:
    def __init__(self, layers: Sequence[B.Layer], max_tokens: int, sink_tokens: int = 4, buffer_tokens: int = 128,
                 device="cuda", batch: int = 1):
        """max_tokens: per sequence.  With batch == 1 the calls take and return tensors without the batch dimension."""
        if buffer_tokens < 1 or sink_tokens < 0 or batch < 1:
            raise ValueError("buffer_tokens >= 1, sink_tokens >= 0 and batch >= 1")
        self.layers = list(layers)
        self.sink_tokens, self.buffer_tokens, self.max_tokens, self.batch = sink_tokens, buffer_tokens, max_tokens, batch
        lay0 = next(l for l in self.layers if l is not None)
        H, g, dt = lay0.kv_heads, lay0.head_dim, lay0.dtype
        self._H, self._g, self._dt = H, g, dt
        raw = lambda *shape: torch.empty(*shape, H, g, dtype=dt, device=device)
        S = max(sink_tokens, 1)
        self.sink = [(raw(batch, S), raw(batch, S)) for _ in self.layers]
        self.buf = [(raw(batch, buffer_tokens), raw(batch, buffer_tokens)) for _ in self.layers]
        cap = max(max_tokens - sink_tokens, 0) // buffer_tokens * buffer_tokens      # the compressed range grows by whole buffers
        self.capacity = cap
        C = max(cap, 1)
        self._C = C
        # sequence b owns tokens [b * C, (b + 1) * C) of the code tensors (and of the 16-bit tensors of a layer given as None)
        self.codes = [None if l is None else (l.alloc_codes(batch * C, device), l.alloc_codes(batch * C, device))
                      for l in self.layers]
        self.raw = [(raw(batch * C), raw(batch * C)) if l is None else None for l in self.layers]
        coded = [l for l in self.layers if l is not None]
        biggest = lambda make: max((make(l) for l in coded), key=lambda t: t.numel())
        # flush: reconstructions of the flushed tokens, two ping-pong pairs (layer l - 1 feeds layer l); with several
        # sequences also the gathered buffers and the codes before they are scattered to their sequences
        R = batch * buffer_tokens
        self._flush_hat = [(raw(R), raw(R)) for _ in range(2)]
        self._flush_ws = biggest(lambda l: l.alloc_workspace(R, device))
        self._flush_in = [(raw(R), raw(R)) for _ in range(2)] if batch > 1 else None
        self._flush_codes = [None if l is None or batch == 1 else (l.alloc_codes(R, device), l.alloc_codes(R, device))
                             for l in self.layers]
        # recovery: [sinks | compressed | buffer] of one layer and sequence (sweep), or the compressed ranges of a
        # group of sequences (attend): two ping-pong pairs
        self._view = [(raw(max(max_tokens, batch * C)), raw(max(max_tokens, batch * C))) for _ in range(2)]
        self._view_ws = biggest(lambda l: l.alloc_workspace(batch * C, device))
        self._group_codes = [None if l is None or batch == 1 else (l.alloc_codes(batch * C, device), l.alloc_codes(batch * C, device))
                             for l in self.layers]
        self._ns, self._nc, self._nb = [0] * batch, [0] * batch, [0] * batch
        self._attend = None                 # buffers of attend(), sized on first use (they depend on the query heads)
        self._device = device

    # ------------------------------------------------------------------ counts
    def _count(self, per_seq: List[int]):
        return per_seq[0] if self.batch == 1 else tuple(per_seq)

    @property
    def n_sink(self):
        return self._count(self._ns)

    @property
    def n_compressed(self):
        return self._count(self._nc)

    @property
    def n_buffered(self):
        return self._count(self._nb)

    @property
    def n_tokens(self):
        return self._count([s + c + b for s, c, b in zip(self._ns, self._nc, self._nb)])

    # ------------------------------------------------------------------ append / flush
    def append(self, kv: Sequence[Tuple[torch.Tensor, torch.Tensor]], lengths: Optional[Sequence[int]] = None) -> None:
        """kv[l] = (K, V) of the new tokens at layer l in the storage dtype: [t, kv_heads, head_dim] for a single
        sequence, [batch, t, kv_heads, head_dim] otherwise; `lengths[b]` <= t tokens of sequence b are taken
        (default: all t)."""
        if len(kv) != len(self.layers):
            raise ValueError("one (K, V) pair per layer")
        if kv[0][0].dim() == 3:
            if self.batch != 1:
                raise ValueError("a batched cache takes [batch, t, kv_heads, head_dim]")
            kv = [(K[None], V[None]) for K, V in kv]
        t = kv[0][0].shape[1]
        n = [t] * self.batch if lengths is None else [int(x) for x in lengths]
        if len(n) != self.batch or kv[0][0].shape[0] != self.batch or any(x < 0 or x > t for x in n):
            raise ValueError("one length per sequence, each at most the tokens given")
        if any(self._ns[b] + self._nc[b] + self._nb[b] + n[b] > self.max_tokens for b in range(self.batch)):
            raise ValueError("cache is full")
        pos = [0] * self.batch
        while True:
            for b in range(self.batch):
                while pos[b] < n[b] and self._nb[b] < self.buffer_tokens:
                    if self._ns[b] < self.sink_tokens:
                        take = min(self.sink_tokens - self._ns[b], n[b] - pos[b])
                        dst, at = self.sink, self._ns[b]
                        self._ns[b] += take
                    else:
                        take = min(self.buffer_tokens - self._nb[b], n[b] - pos[b])
                        dst, at = self.buf, self._nb[b]
                        self._nb[b] += take
                    for l, (K, V) in enumerate(kv):
                        dst[l][0][b, at:at + take].copy_(K[b, pos[b]:pos[b] + take])
                        dst[l][1][b, at:at + take].copy_(V[b, pos[b]:pos[b] + take])
                    pos[b] += take
            full = [b for b in range(self.batch) if self._nb[b] == self.buffer_tokens]
            if not full:
                break
            self._flush(full)

    def _flush(self, full: List[int]) -> None:
        """The full buffers of the sequences `full` are quantized together from the first layer to the last; each
        sequence's codes land behind its own compressed range."""
        r, C, n = self.buffer_tokens, self._C, len(full)
        single = self.batch == 1
        if not single:
            dest = torch.cat([torch.arange(b * C + self._nc[b], b * C + self._nc[b] + r) for b in full]).to(self._device)
            whole = n == self.batch                          # the buffers of all sequences are one contiguous tensor
            pick = None if whole else torch.tensor(full, device=self._device)
        Kp = Vp = None
        for l, lay in enumerate(self.layers):
            if single:
                Xk, Xv = self.buf[l][0][0], self.buf[l][1][0]
            elif whole:
                Xk, Xv = self.buf[l][0].view(n * r, self._H, self._g), self.buf[l][1].view(n * r, self._H, self._g)
            else:
                Xk, Xv = (t[:n * r] for t in self._flush_in[l & 1])
                torch.index_select(self.buf[l][0], 0, pick, out=Xk.view(n, r, self._H, self._g))
                torch.index_select(self.buf[l][1], 0, pick, out=Xv.view(n, r, self._H, self._g))
            if lay is None:                                  # kept in 16 bits: stored as is, feeds the next layer exactly
                if single:
                    at = self._nc[0]
                    self.raw[l][0][at:at + r].copy_(Xk); self.raw[l][1][at:at + r].copy_(Xv)
                    Kp, Vp = self.raw[l][0][at:at + r], self.raw[l][1][at:at + r]
                else:
                    self.raw[l][0].index_copy_(0, dest, Xk); self.raw[l][1].index_copy_(0, dest, Xv)
                    Kp, Vp = Xk, Xv
                continue
            (kc, ks), (vc, vs) = self.codes[l]
            Kh, Vh = (t[:n * r] for t in self._flush_hat[l & 1])
            if single:
                at = self._nc[0]
                out = (kc[at:at + r], ks[at:at + r], vc[at:at + r], vs[at:at + r])
            else:
                (skc, sks), (svc, svs) = self._flush_codes[l]
                out = (skc[:n * r], sks[:n * r], svc[:n * r], svs[:n * r])
            B.aquakv_encode_layer(lay, n * r, Xk, Xv, Kp, Vp, *out, Kh, Vh, self._flush_ws)
            if not single:
                for store, staged in zip((kc, ks, vc, vs), out):
                    store.index_copy_(0, dest, staged)
            Kp, Vp = Kh, Vh
        for b in full:
            self._nc[b] += r
            self._nb[b] = 0

    # ------------------------------------------------------------------ recovery of one sequence
    def sweep(self, seq: int = 0) -> Iterator[Tuple[int, torch.Tensor, torch.Tensor]]:
        """Yield (layer, K, V) of sequence `seq` for every layer in order, K and V being [n_tokens, kv_heads,
        head_dim]: sinks, the recovered compressed past, the buffered tokens.  The tensors are views of two
        ping-pong buffers: layer l's are valid until layer l + 2 is produced."""
        s, c, b = self._ns[seq], self._nc[seq], self._nb[seq]
        at = seq * self._C
        Kp = Vp = None
        for l, lay in enumerate(self.layers):
            K, V = self._view[l & 1]
            if s:
                K[:s].copy_(self.sink[l][0][seq, :s]); V[:s].copy_(self.sink[l][1][seq, :s])
            if c and lay is None:
                K[s:s + c].copy_(self.raw[l][0][at:at + c]); V[s:s + c].copy_(self.raw[l][1][at:at + c])
                Kp, Vp = K[s:s + c], V[s:s + c]
            elif c:
                (kc, ks), (vc, vs) = self.codes[l]
                B.aquakv_decode_layer(lay, c, kc[at:at + c], ks[at:at + c], vc[at:at + c], vs[at:at + c], Kp, Vp,
                                      K[s:s + c], V[s:s + c], self._view_ws)
                Kp, Vp = K[s:s + c], V[s:s + c]
            if b:
                K[s + c:s + c + b].copy_(self.buf[l][0][seq, :b]); V[s + c:s + c + b].copy_(self.buf[l][1][seq, :b])
            yield l, K[:s + c + b], V[:s + c + b]

    # ------------------------------------------------------------------ attention of one new token per sequence
    def attend(self, queries: Sequence[torch.Tensor], score_scale: float, rope=None) -> List[torch.Tensor]:
        """queries[l]: the new token's queries at layer l in the storage dtype, [q_heads, head_dim] for a single
        sequence, [batch, q_heads, head_dim] otherwise.  Returns one fp32 tensor of the same shape per layer:
        softmax(score_scale * q K^T) V over sinks, compressed past and buffer of the query's own sequence.
        One sweep over the layers per group of sequences with equally long compressed ranges; the recovered tensors
        of layer l feed layer l + 1 as in `sweep`.
        rope = (cos, sin), device fp32 [>= n_tokens, head_dim / 2]: the cache holds keys from before the rotary
        embedding (Sect. 3.3, the paper's default); the key of token t of a sequence is rotated by row t on the fly,
        the queries are taken as already rotated, and what is recovered for the next layer stays unrotated."""
        if any(s + c + b == 0 for s, c, b in zip(self._ns, self._nc, self._nb)):
            raise ValueError("nothing cached")
        H, g, dt, NB = self._H, self._g, self._dt, self.batch
        single = queries[0].dim() == 2
        if single and NB != 1:
            raise ValueError("a batched cache takes [batch, q_heads, head_dim]")
        qs = [q[None] if single else q for q in queries]
        QH = qs[0].shape[1]
        if self._attend is None or self._attend["q_heads"] != QH:
            coded = [l for l in self.layers if l is not None]
            self._attend = dict(
                q_heads=QH,
                scores=torch.empty(NB * QH * self._C, dtype=torch.float32, device=self._device),
                out=[torch.empty(NB, QH, g, dtype=torch.float32, device=self._device) for _ in self.layers],
                group_out=torch.empty(NB, QH, g, dtype=torch.float32, device=self._device),
                group_q=torch.empty(NB, QH, g, dtype=dt, device=self._device),
                stats=torch.empty(NB, QH, 2, dtype=torch.float32, device=self._device),
                ws=max((l.alloc_weighted_workspace(NB, self._C, QH, self._device) for l in coded), key=lambda t: t.numel()))
        A = self._attend
        step = 4096                                              # tokens per aquakv_attend_raw call
        cos, sin = rope if rope is not None else (None, None)
        rows = lambda t, a, n: None if t is None else t[a:a + n]  # the angles of tokens a ... a + n - 1
        C = self._C
        groups: Dict[int, List[int]] = {}
        for b in range(NB):
            groups.setdefault(self._nc[b], []).append(b)
        for c, members in groups.items():
            n = len(members)
            direct = n == 1                                      # one sequence: its own ranges, nothing is gathered
            in_place = members == list(range(NB))                # the whole batch in order: results need no scatter
            first = members[0] * C
            s0 = self._ns[members[0]]                            # compressed tokens exist only behind full sinks
            Kp = Vp = None
            for l, lay in enumerate(self.layers):
                q = qs[l] if in_place else A["group_q"][:n]
                if not in_place:
                    for i, b in enumerate(members):
                        q[i].copy_(qs[l][b])
                out = A["out"][l] if in_place else A["group_out"][:n]
                stats = A["stats"][:n]
                have = False
                K, V = (t[:n * c] for t in self._view[l & 1])
                if c and lay is None:                            # compressed range kept in 16 bits
                    for i, b in enumerate(members):
                        Kb, Vb = self.raw[l][0][b * C:b * C + c], self.raw[l][1][b * C:b * C + c]
                        for r0 in range(0, c, step):
                            m = min(step, c - r0)
                            B.aquakv_attend_raw(dt, 1, m, H, QH, Kb[r0:r0 + m], Vb[r0:r0 + m], q[i:i + 1], score_scale,
                                                out[i:i + 1], stats[i:i + 1], r0 > 0,
                                                rope_cos=rows(cos, s0 + r0, m), rope_sin=rows(sin, s0 + r0, m))
                        if not direct:
                            K[i * c:(i + 1) * c].copy_(Kb); V[i * c:(i + 1) * c].copy_(Vb)
                    Kp, Vp = (self.raw[l][0][first:first + c], self.raw[l][1][first:first + c]) if direct else (K, V)
                    have = True
                elif c:
                    (kc, ks), (vc, vs) = self.codes[l]
                    if direct:
                        kc, ks, vc, vs = (t[first:first + c] for t in (kc, ks, vc, vs))
                    else:
                        staged = [t[:n * c] for pair in self._group_codes[l] for t in pair]
                        for i, b in enumerate(members):
                            for dst, src in zip(staged, (kc, ks, vc, vs)):
                                dst[i * c:(i + 1) * c].copy_(src[b * C:b * C + c])
                        kc, ks, vc, vs = staged
                    scores = A["scores"][:n * QH * c].view(n, QH, c)
                    if rope is None:
                        B.aquakv_decode_attn_scores(lay, n, c, QH, kc, ks, Kp, q, score_scale, scores, K, self._view_ws)
                    else:
                        B.aquakv_decode_attn_scores_rope(lay, n, c, QH, kc, ks, Kp, q, rows(cos, s0, c), rows(sin, s0, c),
                                                         score_scale, scores, K, self._view_ws)
                    B.aquakv_decode_values_attend(lay, n, c, QH, vc, vs, Vp, K, scores, V, out, stats, A["ws"])
                    Kp, Vp = K, V
                    have = True
                for i, b in enumerate(members):
                    s, nb = self._ns[b], self._nb[b]
                    mine = have
                    if s:
                        B.aquakv_attend_raw(dt, 1, s, H, QH, self.sink[l][0][b, :s], self.sink[l][1][b, :s], q[i:i + 1],
                                            score_scale, out[i:i + 1], stats[i:i + 1], mine,
                                            rope_cos=rows(cos, 0, s), rope_sin=rows(sin, 0, s))
                        mine = True
                    for r0 in range(0, nb, step):
                        m = min(step, nb - r0)
                        B.aquakv_attend_raw(dt, 1, m, H, QH, self.buf[l][0][b, r0:r0 + m], self.buf[l][1][b, r0:r0 + m],
                                            q[i:i + 1], score_scale, out[i:i + 1], stats[i:i + 1], mine,
                                            rope_cos=rows(cos, s + c + r0, m), rope_sin=rows(sin, s + c + r0, m))
                        mine = True
                if not in_place:
                    for i, b in enumerate(members):
                        A["out"][l][b].copy_(out[i])
        return [o[0] if single else o for o in A["out"]]

    def stored_bytes(self) -> int:
        """Bytes the cache content occupies (all layers, all sequences): 16-bit sinks and buffer, packed codes and
        fp16 scales."""
        lay0 = next(l for l in self.layers if l is not None)
        per_tok = lay0.d * self.sink[0][0].element_size() * 2
        total = (sum(self._ns) + sum(self._nb)) * per_tok * len(self.layers)
        n_compressed = sum(self._nc)
        for lay in self.layers:
            if lay is None:
                total += n_compressed * per_tok
                continue
            groups = lay.d // lay.rht_group
            total += 2 * n_compressed * (lay.kv_heads * lay.code_bytes_per_group + 2 * groups * lay.scale_words_per_group)
        return total
