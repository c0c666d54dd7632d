"""CPU oracle for one retraining step of a learned cache.  TEST INFRASTRUCTURE ONLY.

Plain numpy in fp64, written from the paper's description of how predictor and selector are
trained (Section 3, "Training Learned Caches") and retrained online (Section 5, "Retraining
Learned Caches"; Section 7 parameters: learning rate 0.002, 5 epochs).  The paper gives the
ingredients, not the formulas; the reading taken here:

  predictor  global pool -> FC(C->H) -> ReLU -> FC(H->K) -> softmax q.
             The section describes a distillation-style loss that uses both the true label and the
             base DNN's class distribution, and prints no formula.  This oracle's reading:
                 t_i = (1 - alpha) * onehot(y_i) + alpha * Y_i        (Y = the base DNN's distribution)
                 L_p = -(1/n) sum_i sum_k t_ik log q_ik
  selector   ground truth G_i = [argmax_k z_ik == argmax_k Y_ik] (the paper's G); the section asks for
             false positives to cost more than false negatives and gives no weight.  This oracle's
             reading, a cross-entropy whose G = 0 term is scaled by fp_weight >= 1:
                 c_i = logistic(ws . [p_i ; q_i] + bs)
                 L_s = -(1/n) sum_i [ G_i log c_i + fp_weight (1 - G_i) log(1 - c_i) ]
             The selector is trained on the predictor's outputs as data: no gradient flows from L_s
             into the predictor.
  update     plain SGD, theta <- theta - lr * grad, both networks in the same step, the selector
             on the predictor's outputs of BEFORE the update.

  Pool(h) predictor (Section 3, table of predictor architectures: pooled windows -> one FC): weights
             without "W1"/"b1"; `pooled` are then the ReLU'd window means and z = W2 pooled + b2.
  hidden-layer selector (Section 3, "Selector Network Design": the paper's selector has one hidden
             layer): when the weights hold "Ws", "cs", "vs" the selector is
                 g_i = relu(Ws [p_i ; q_i] + cs),  c_i = logistic(vs . g_i + bs)
             with the same loss; its gradients flow through the ReLU into Ws and cs, never into q.

  FC(h) predictor (same table: the flattened hidden-layer output -> FC(D->H) -> ReLU -> FC(H->K)): the same
             two-layer network with `pooled` = the flattened rows; the selector reads [h ; q], the hidden
             layer and the class distribution, as the lookup does (`sel_input="hidden"`).  The hidden layer
             is data to the selector, like q: no gradient flows from L_s into the predictor.
  Conv(k,s) predictor (same table: Input -Conv-> Hidden -FC-> Output): weights with a 4-d "W1"
             [filters, C, k, k]; `pooled` is the map [n, C, in_h, in_w]; a = conv(x, W1, stride s, no padding)
             + b1 per filter, h = relu(a) flattened [filter][oy][ox]; the selector reads [h ; q].
  softmax-threshold mode (the paper's ablation without a selector network): weights with neither "ws" nor
             "Ws"; only the predictor is trained, L_s = 0.

Every function takes and returns fp64 arrays; `pooled` are the features the lookup oracle reports (the
flattened rows / the map for the last two predictors).  `arch` holds what the weights do not say:
{"sel_input": "input" | "hidden", "stride": s}.
"""
from __future__ import annotations

import numpy as np


def _windows(x: np.ndarray, k: int, s: int) -> np.ndarray:
    """[n, C, oh, ow, k, k] view of the k x k windows of x [n, C, ih, iw] at stride s, no padding."""
    v = np.lib.stride_tricks.sliding_window_view(x, (k, k), axis=(2, 3))
    return v[:, :, ::s, ::s]


def forward(w: dict, pooled: np.ndarray, arch: dict = None):
    arch = arch or {}
    p = np.asarray(pooled, np.float64)
    W2, b2 = np.asarray(w["W2"], np.float64), np.asarray(w["b2"], np.float64)
    out = {}
    if "W1" in w and np.ndim(w["W1"]) == 4:
        W1 = np.asarray(w["W1"], np.float64)
        win = _windows(p, W1.shape[2], int(arch.get("stride", 1)))
        a = np.einsum("ncyxij,ocij->noyx", win, W1) + np.asarray(w["b1"], np.float64)[None, :, None, None]
        out["win"] = win
        out["a4"] = a
        a = a.reshape(len(p), -1)                       # [filter][oy][ox]
        h = np.maximum(a, 0.0)
        feats = h
    elif "W1" in w:
        a = p @ np.asarray(w["W1"], np.float64).T + np.asarray(w["b1"], np.float64)
        h = np.maximum(a, 0.0)
        feats = h if arch.get("sel_input", "input") == "hidden" else p
    else:                         # Pool(h): the (already ReLU'd) pooled windows feed the output layer directly
        a = h = p
        feats = p
    z = h @ W2.T + b2
    e = np.exp(z - z.max(axis=1, keepdims=True))
    q = e / e.sum(axis=1, keepdims=True)
    x = np.concatenate([feats, q], axis=1)              # what the selector reads
    out.update({"p": p, "a": a, "h": h, "z": z, "q": q, "x": x})
    if "Ws" in w:
        sa = x @ np.asarray(w["Ws"], np.float64).T + np.asarray(w["cs"], np.float64)
        g = np.maximum(sa, 0.0)
        u = g @ np.asarray(w["vs"], np.float64) + float(w["bs"])
        out.update({"sa": sa, "g": g})
    elif "ws" in w:
        u = x @ np.asarray(w["ws"], np.float64) + float(w["bs"])
    else:                         # no selector network
        u = None
    out["u"] = u
    out["c"] = None if u is None else 1.0 / (1.0 + np.exp(-u))
    return out


def targets(labels: np.ndarray, teacher: np.ndarray, alpha: float) -> np.ndarray:
    Y = np.asarray(teacher, np.float64)
    t = alpha * Y
    t[np.arange(len(labels)), np.asarray(labels)] += 1.0 - alpha
    return t


def losses(w: dict, pooled, labels, teacher, alpha: float, fp_weight: float, arch: dict = None):
    f = forward(w, pooled, arch)
    n = len(labels)
    t = targets(labels, teacher, alpha)
    logq = f["z"] - f["z"].max(axis=1, keepdims=True)
    logq = logq - np.log(np.exp(logq).sum(axis=1, keepdims=True))
    Lp = -float((t * logq).sum()) / n
    if f["u"] is None:
        return Lp, 0.0
    G = (f["z"].argmax(axis=1) == np.asarray(teacher).argmax(axis=1)).astype(np.float64)
    # log c and log(1-c) from u, stable for large |u|
    log_c = -np.logaddexp(0.0, -f["u"])
    log_1mc = -np.logaddexp(0.0, f["u"])
    Ls = -float((G * log_c + fp_weight * (1.0 - G) * log_1mc).sum()) / n
    return Lp, Ls


def gradients(w: dict, pooled, labels, teacher, alpha: float, fp_weight: float, arch: dict = None) -> dict:
    f = forward(w, pooled, arch)
    n = len(labels)
    t = targets(labels, teacher, alpha)
    dz = (f["q"] - t) / n
    W2 = np.asarray(w["W2"], np.float64)
    dW2 = dz.T @ f["h"]
    db2 = dz.sum(axis=0)
    out = {"W2": dW2, "b2": db2}
    if "W1" in w:
        dh = (dz @ W2) * (f["a"] > 0.0)
        if np.ndim(w["W1"]) == 4:
            da = dh.reshape(f["a4"].shape)
            out["W1"] = np.einsum("noyx,ncyxij->ocij", da, f["win"])
            out["b1"] = da.sum(axis=(0, 2, 3))
        else:
            out["W1"] = dh.T @ f["p"]
            out["b1"] = dh.sum(axis=0)
    if f["u"] is None:
        return out
    G = (f["z"].argmax(axis=1) == np.asarray(teacher).argmax(axis=1)).astype(np.float64)
    du = (G * (f["c"] - 1.0) + fp_weight * (1.0 - G) * f["c"]) / n
    out["bs"] = float(du.sum())
    if "Ws" in w:
        dg = np.outer(du, np.asarray(w["vs"], np.float64)) * (f["sa"] > 0.0)
        out.update({"vs": du @ f["g"], "Ws": dg.T @ f["x"], "cs": dg.sum(axis=0)})
    else:
        out["ws"] = du @ f["x"]
    return out


def sgd_step(w: dict, pooled, labels, teacher, lr: float, alpha: float, fp_weight: float, arch: dict = None):
    """One step on one batch.  Returns (new weights as fp64 arrays, predictor loss, selector loss),
    the losses evaluated before the update."""
    g = gradients(w, pooled, labels, teacher, alpha, fp_weight, arch)
    Lp, Ls = losses(w, pooled, labels, teacher, alpha, fp_weight, arch)
    new = {k: np.asarray(w[k], np.float64) - lr * g[k] for k in g if k != "bs"}
    if "bs" in g:
        new["bs"] = float(w["bs"]) - lr * g["bs"]
    return new, Lp, Ls
