"""CPU oracle of predictor calibration.

TEST INFRASTRUCTURE ONLY (same rules as aquakv_oracle.py: imported by tests only, shares no code with the product
package).

What it follows (AQUA-KV paper, arxiv 2501.19392):
  * Sect. 3.2: the predictors are linear regressions, trained one layer at a time, each set on the previous layer's
    *reconstructed* keys / values, because reconstructions are what the predictors will see at inference time.
  * Alg. "Calibration": per layer, f_key = argmin || f(K_old) - K ||^2; K_rec = f_key(K_old) + Q^-1(Q(K - f_key(K_old)));
    f_value = argmin || f([V_old; K_rec]) - V ||^2; V_rec likewise; then (K_old, V_old) <- (K_rec, V_rec).

Readings taken where the paper is silent or at odds with itself:
  * The least-squares problem is solved through its normal equations with a ridge term,
    W = (X^T X + lambda I)^-1 X^T Y, lambda = rate * trace(X^T X) / d_in; rate = 0 is the plain argmin of the
    algorithm (needs X of full column rank).  The appendix gives a regulariser rate of 1e-3 for its linear
    probes without saying relative to what; relative to the mean diagonal of X^T X makes it scale free.
  * The fit has an optional intercept (centred regression; Sect. 4.1 lists a bias-only predictor among its
    ablations, so the predictors carry a bias).  The layer-by-layer procedure here fits none: the synthetic
    workloads have zero-mean channels.
  * The weights are rounded to the storage dtype before they are used to encode the layer: it is the rounded
    predictor that inference runs, so the next layer is fitted on what that predictor reconstructs.
  * The first layer: the algorithm's listing hands its raw K, V to the second layer's fit, the text says the
    first layer goes through the backbone quantizer alone and that predictors see reconstructions.  Here the first layer's entry is a
    Layer without predictors (its reconstruction under that layer's backbone is what the second layer is fitted
    on) or None (kept in 16 bits: the raw tensors, the listing's reading).

Pins (tests/test_calibration.py): exact recovery of a noise-free linear map, the normal-equation residual
X^T (X W^T - Y) + lambda W^T = 0, agreement with numpy's least-squares routine as rate -> 0, the one-dimensional
closed form, shrinkage under the ridge term; for the layer-by-layer procedure: each predictor is the regression on
the reconstructions actually produced, and calibrated predictors cut the reconstruction error of a correlated
stream several-fold (the claim of Sect. 3.1).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import aquakv_oracle as O


def fit_predictor(X, Y, rate: float = 1e-3, bias: bool = False):
    """Ridge least squares through the normal equations.  X [T, d_in], Y [T, d_out] -> W [d_out, d_in] (fp64),
    the layout of Layer.w_k / w_v: prediction = X @ W.T.

    bias = True fits an intercept as well, prediction = X @ W.T + b: the regression of the centred Y on the centred
    X (the ridge term acts on W only, and on the centred Gram matrix), b = mean(Y) - W mean(X); returns (W, b)."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    d_in = X.shape[1]
    if bias:
        mx, my = X.mean(axis=0), Y.mean(axis=0)
        X, Y = X - mx, Y - my
    G = X.T @ X
    lam = rate * np.trace(G) / d_in
    W = np.linalg.solve(G + lam * np.eye(d_in), X.T @ Y).T
    return (W, my - W @ mx) if bias else W


def calibrate(layers: Sequence[Optional[O.Layer]], Ks: Sequence[np.ndarray], Vs: Sequence[np.ndarray],
              rate: float = 1e-3) -> Tuple[List[Optional[O.Layer]], List[dict]]:
    """Alg. "Calibration" on given per-layer tensors Ks[l], Vs[l] [T, H, g] (storage-dtype values).

    layers[l] carries the backbone of layer l (grid, signs, dtype); its predictor fields are ignored and replaced.
    layers[0] may be None (first layer kept in 16 bits).  Returns the layers with fitted, storage-rounded
    predictors (layer 0 unchanged) and, per layer, the reconstructions the next layer was fitted on."""
    out: List[Optional[O.Layer]] = []
    trace: List[dict] = []
    K_old = V_old = None
    for l, lay in enumerate(layers):
        K = np.asarray(Ks[l], dtype=np.float64)
        V = np.asarray(Vs[l], dtype=np.float64)
        T = K.shape[0]
        if l == 0:
            if lay is None:
                K_old, V_old = K, V
                out.append(None)
            else:
                first = dataclasses.replace(lay, w_k=None, b_k=None, w_v=None, b_v=None)
                e = O.encode_layer(first, K, V)
                K_old, V_old = e["Khat"], e["Vhat"]
                out.append(first)
            trace.append(dict(Khat=K_old, Vhat=V_old))
            continue
        w_k = O.round_storage(fit_predictor(K_old.reshape(T, -1), K.reshape(T, -1), rate), lay.dtype)
        keyed = dataclasses.replace(lay, w_k=w_k, b_k=None, w_v=None, b_v=None)
        K_rec = O.encode_layer(keyed, K, V, K_old, None)["Khat"]            # V side unused here (no value predictor yet)
        x_v = np.concatenate([V_old.reshape(T, -1), K_rec.reshape(T, -1)], axis=1)
        w_v = O.round_storage(fit_predictor(x_v, V.reshape(T, -1), rate), lay.dtype)
        full = dataclasses.replace(lay, w_k=w_k, b_k=None, w_v=w_v, b_v=None)
        e = O.encode_layer(full, K, V, K_old, V_old)
        assert np.array_equal(e["Khat"], K_rec)
        K_old, V_old = e["Khat"], e["Vhat"]
        out.append(full)
        trace.append(dict(Khat=K_old, Vhat=V_old))
    return out, trace
