"""The scoring call for callers that cannot allocate (aquakv_decode_attn_scores_folded_static: the folded queries live
in a buffer built into the library) against aquakv_decode_attn_scores_folded with a caller's workspace: same kernels,
so the same bits, on two calls in a row into the one built-in buffer, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2501_19392_amd import synth
from tests import parity_utils as U

pytestmark = pytest.mark.gpu


def _cache(lg, T, seed):
    """Random content of a compressed key cache (the scoring call takes any codes): codes, scales, Khat_prev."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    kc, ks = lg.alloc_codes(T)
    kc.copy_(torch.randint(0, 256, kc.shape, generator=gen, device="cuda", dtype=torch.int32).to(torch.uint8))
    ks.copy_((torch.rand(ks.shape, generator=gen, device="cuda") * 2 + 0.05).half().view(torch.int16))
    Kprev = torch.randn(T, lg.kv_heads, 128, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    return kc, ks, Kprev


def test_built_in_buffer_gives_the_bits_of_the_workspace_call():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests must run on an MI355X")
    from paper_2501_19392_amd import binding as B
    H = 8
    bk = torch.randn(1024, generator=torch.Generator().manual_seed(5)) * 0.3
    _, lg = U.make_layers(H, "bf16", 16, layer_idx=2, w_k=U.random_weights(1024, 1024, 3, 0.7),
                          w_v=U.random_weights(1024, 2048, 4, 0.7), b_k=bk)
    # first a large call (two passes: 64 query heads, ragged last tile), then a smaller one (one pass, fewer sequences,
    # fewer heads), then the large one again: nothing of an earlier call may show in a later one
    shapes = [(5, 1000, 64, 11), (2, 70, 24, 12), (5, 1000, 64, 11)]
    for batch, S, QH, seed in shapes:
        print(f"case built-in buffer batch={batch} S={S} QH={QH}", flush=True)
        T = batch * S
        kc, ks, Kprev = _cache(lg, T, synth.BASE_SEED + seed)
        q = synth.random_queries(batch, QH, 128, seed=seed, dtype="bf16", device="cuda")
        want = torch.full((batch, QH, S), float("nan"), dtype=torch.float32, device="cuda")
        B.aquakv_decode_attn_scores_folded(lg, batch, S, QH, kc, ks, Kprev, q, 0.0883883, want, lg.alloc_scores_workspace(batch, QH))
        got = torch.full((batch, QH, S), float("nan"), dtype=torch.float32, device="cuda")
        B.aquakv_decode_attn_scores_folded_static(lg, batch, S, QH, kc, ks, Kprev, q, 0.0883883, got)
        torch.cuda.synchronize()
        assert torch.isfinite(want).all()
        assert torch.equal(got.view(torch.int32), want.view(torch.int32))
    # beyond the built-in buffer: refused with a text, nothing launched
    with pytest.raises(B.AquaKVError) as e:
        B.aquakv_decode_attn_scores_folded_static(lg, 65, 8, 32, kc, ks, Kprev, q, 1.0, got)
    assert e.value.status == B.AQUAKV_EUNSUPPORTED and "aquakv_decode_attn_scores_folded" in str(e.value)
    _ = np
