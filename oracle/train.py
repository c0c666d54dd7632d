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

Every function takes and returns fp64 arrays; `pooled` are the features the lookup oracle reports.
"""
from __future__ import annotations

import numpy as np


def forward(w: dict, pooled: np.ndarray):
    p = np.asarray(pooled, np.float64)
    W2, b2 = np.asarray(w["W2"], np.float64), np.asarray(w["b2"], np.float64)
    if "W1" in w:
        a = p @ np.asarray(w["W1"], np.float64).T + np.asarray(w["b1"], np.float64)
        h = np.maximum(a, 0.0)
    else:                         # Pool(h): the (already ReLU'd) pooled windows feed the output layer directly
        a = h = p
    z = h @ W2.T + b2
    e = np.exp(z - z.max(axis=1, keepdims=True))
    q = e / e.sum(axis=1, keepdims=True)
    x = np.concatenate([p, q], axis=1)
    out = {"p": p, "a": a, "h": h, "z": z, "q": q, "x": x}
    if "Ws" in w:
        sa = x @ np.asarray(w["Ws"], np.float64).T + np.asarray(w["cs"], np.float64)
        g = np.maximum(sa, 0.0)
        u = g @ np.asarray(w["vs"], np.float64) + float(w["bs"])
        out.update({"sa": sa, "g": g})
    else:
        u = x @ np.asarray(w["ws"], np.float64) + float(w["bs"])
    out["u"] = u
    out["c"] = 1.0 / (1.0 + np.exp(-u))
    return out


def targets(labels: np.ndarray, teacher: np.ndarray, alpha: float) -> np.ndarray:
    Y = np.asarray(teacher, np.float64)
    t = alpha * Y
    t[np.arange(len(labels)), np.asarray(labels)] += 1.0 - alpha
    return t


def losses(w: dict, pooled, labels, teacher, alpha: float, fp_weight: float):
    f = forward(w, pooled)
    n = len(labels)
    t = targets(labels, teacher, alpha)
    logq = f["z"] - f["z"].max(axis=1, keepdims=True)
    logq = logq - np.log(np.exp(logq).sum(axis=1, keepdims=True))
    Lp = -float((t * logq).sum()) / n
    G = (f["z"].argmax(axis=1) == np.asarray(teacher).argmax(axis=1)).astype(np.float64)
    # log c and log(1-c) from u, stable for large |u|
    log_c = -np.logaddexp(0.0, -f["u"])
    log_1mc = -np.logaddexp(0.0, f["u"])
    Ls = -float((G * log_c + fp_weight * (1.0 - G) * log_1mc).sum()) / n
    return Lp, Ls


def gradients(w: dict, pooled, labels, teacher, alpha: float, fp_weight: float) -> dict:
    f = forward(w, pooled)
    n = len(labels)
    t = targets(labels, teacher, alpha)
    dz = (f["q"] - t) / n
    W2 = np.asarray(w["W2"], np.float64)
    dW2 = dz.T @ f["h"]
    db2 = dz.sum(axis=0)
    if "W1" in w:
        dh = (dz @ W2) * (f["a"] > 0.0)
        dW1 = dh.T @ f["p"]
        db1 = dh.sum(axis=0)
    G = (f["z"].argmax(axis=1) == np.asarray(teacher).argmax(axis=1)).astype(np.float64)
    du = (G * (f["c"] - 1.0) + fp_weight * (1.0 - G) * f["c"]) / n
    out = {"W2": dW2, "b2": db2, "bs": float(du.sum())}
    if "W1" in w:
        out.update({"W1": dW1, "b1": db1})
    if "Ws" in w:
        dg = np.outer(du, np.asarray(w["vs"], np.float64)) * (f["sa"] > 0.0)
        out.update({"vs": du @ f["g"], "Ws": dg.T @ f["x"], "cs": dg.sum(axis=0)})
    else:
        out["ws"] = du @ f["x"]
    return out


def sgd_step(w: dict, pooled, labels, teacher, lr: float, alpha: float, fp_weight: float):
    """One step on one batch.  Returns (new weights as fp64 arrays, predictor loss, selector loss),
    the losses evaluated before the update."""
    g = gradients(w, pooled, labels, teacher, alpha, fp_weight)
    Lp, Ls = losses(w, pooled, labels, teacher, alpha, fp_weight)
    new = {k: np.asarray(w[k], np.float64) - lr * g[k] for k in g if k != "bs"}
    new["bs"] = float(w["bs"]) - lr * g["bs"]
    return new, Lp, Ls
