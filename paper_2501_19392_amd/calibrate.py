"""Layer-by-layer calibration of the predictors over the C-ABI calls.

AQUA-KV paper (arxiv 2501.19392), Sect. 3.2 and Alg. "Calibration": the predictors are trained one layer at a time,
each on the previous layer's *reconstructed* keys / values: fit f_key on (Khat_prev, K), encode the keys with it,
fit f_value on ([Vhat_prev ; Khat], V), encode the values, move on.  The first layer has no predictor: it is either
quantized by its backbone alone (its reconstruction feeds the second layer's fit) or kept in 16 bits (passed as None:
the raw tensors feed it).

Bookkeeping only: the fits run in `aquakv_fit_predictor`, the reconstructions come from `aquakv_encode_keys` /
`aquakv_encode_values`; torch tensors are the device memory they work on.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence, Tuple

import torch

from . import binding as B


def calibrate(make_layer: Callable[..., Optional[B.Layer]], n_layers: int, kv: Callable[[int], Tuple[torch.Tensor, torch.Tensor]],
              rate: float = 1e-3, device="cuda") -> List[Optional[B.Layer]]:
    """make_layer(l, w_k=None, w_v=None) builds layer l's `Layer` (backbone: grid, signs, dtype) with the given
    predictor weights; make_layer(0) may return None (first layer kept in 16 bits).  kv(l) returns (K, V) of layer l,
    [tokens, kv_heads, head_dim] in the storage dtype on `device` (called once per layer, in order, so a caller can
    stream them).  Returns the layers with fitted predictors."""
    out: List[Optional[B.Layer]] = []
    K_old = V_old = None
    fit_ws = None
    for l in range(n_layers):
        K, V = kv(l)
        T, H, g = K.shape
        D = H * g
        if l == 0:
            lay = make_layer(0)
            if lay is None:
                K_old, V_old = K, V
            else:
                K_old, V_old = lay.alloc_kv(T, device), lay.alloc_kv(T, device)
                kc, ks = lay.alloc_codes(T, device)
                vc, vs = lay.alloc_codes(T, device)
                B.aquakv_encode_layer(lay, T, K, V, None, None, kc, ks, vc, vs, K_old, V_old, lay.alloc_workspace(T, device))
            out.append(lay)
            continue
        dt = K.dtype
        if fit_ws is None:
            fit_ws = torch.empty(B.aquakv_fit_workspace_bytes(2 * D, D), dtype=torch.uint8, device=device)
        w_k = torch.empty(D, D, dtype=dt, device=device)
        B.aquakv_fit_predictor(dt, T, K_old, D, None, 0, K, D, rate, w_k, None, fit_ws)
        keyed = make_layer(l, w_k=w_k)
        K_rec = keyed.alloc_kv(T, device)
        kc, ks = keyed.alloc_codes(T, device)
        ws = keyed.alloc_workspace(T, device)
        B.aquakv_encode_keys(keyed, T, K, K_old, kc, ks, K_rec, ws)
        w_v = torch.empty(D, 2 * D, dtype=dt, device=device)
        B.aquakv_fit_predictor(dt, T, V_old, D, K_rec, D, V, D, rate, w_v, None, fit_ws)
        full = make_layer(l, w_k=w_k, w_v=w_v)
        V_rec = full.alloc_kv(T, device)
        vc, vs = full.alloc_codes(T, device)
        B.aquakv_encode_values(full, T, V, V_old, K_rec, vc, vs, V_rec, full.alloc_workspace(T, device))
        out.append(full)
        K_old, V_old = K_rec, V_rec
    return out
