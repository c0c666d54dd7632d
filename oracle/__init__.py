"""CPU oracle for the learned-cache lookup.  TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``gati_oracle.c`` (plain C, fp64 accumulation, one thread)
plus the layer-to-layer loop of a cache stack.  Nothing in the product package
imports this; only tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gati_oracle.c")
_LIB = os.path.join(_HERE, "libgati_oracle.so")

F32, BF16 = 0, 1
NCS, NSC = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math: the fp64 loops stay as written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Desc(C.Structure):
    _fields_ = [("C", C.c_int32), ("S", C.c_int32), ("H", C.c_int32), ("K", C.c_int32),
                ("act_dtype", C.c_int32), ("layout", C.c_int32), ("round_operands", C.c_int32),
                ("threshold", C.c_float), ("selector", C.c_int32), ("predictor", C.c_int32),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("out_h", C.c_int32), ("out_w", C.c_int32),
                ("sel_hidden", C.c_int32), ("conv_k", C.c_int32), ("conv_s", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
                ("ws", C.c_void_p), ("bs", C.c_float),
                ("Ws", C.c_void_p), ("cs", C.c_void_p), ("vs", C.c_void_p)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_round_bf16.restype = C.c_double
        _lib.oracle_round_bf16.argtypes = [C.c_double]
        _lib.oracle_lookup.restype = C.c_int
        _lib.oracle_lookup.argtypes = [C.POINTER(_Desc), C.POINTER(_Weights), C.c_void_p, C.c_void_p,
                                       C.c_int32] + [C.c_void_p] * 7
        _lib.oracle_compact_misses.restype = C.c_int32
        _lib.oracle_compact_misses.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        _lib.oracle_pool_row.restype = None
        _lib.oracle_pool_row.argtypes = [C.POINTER(_Desc), C.c_void_p, C.c_int64, C.c_void_p]
        _lib.oracle_pool_adaptive_row.restype = None
        _lib.oracle_pool_adaptive_row.argtypes = [C.POINTER(_Desc), C.c_void_p, C.c_int64, C.c_void_p]
        _lib.oracle_fc1_relu.restype = C.c_int
        _lib.oracle_fc1_relu.argtypes = [C.POINTER(_Desc), C.POINTER(_Weights), C.c_void_p, C.c_void_p]
        _lib.oracle_fc2.restype = C.c_int
        _lib.oracle_fc2.argtypes = [C.POINTER(_Desc), C.POINTER(_Weights), C.c_void_p, C.c_void_p]
        _lib.oracle_softmax_argmax.restype = C.c_int32
        _lib.oracle_softmax_argmax.argtypes = [C.c_int, C.c_void_p, C.c_void_p]
        _lib.oracle_selector_score.restype = C.c_double
        _lib.oracle_selector_score.argtypes = [C.POINTER(_Desc), C.POINTER(_Weights), C.c_void_p, C.c_void_p]
        _lib.oracle_selector_hidden_score.restype = C.c_double
        _lib.oracle_selector_hidden_score.argtypes = [C.POINTER(_Desc), C.POINTER(_Weights), C.c_void_p, C.c_void_p]
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class CacheDef:
    """Shapes and arithmetic mode of one learned cache, as the oracle sees it."""
    C: int
    S: int
    H: int
    K: int
    dtype: str = "f32"          # activation element type: "f32" | "bf16" (uint16 bit patterns)
    layout: str = "ncs"         # "ncs" | "nsc"
    threshold: float = 0.5
    round_operands: bool = False  # bf16 cache arithmetic (see gati_oracle.c)
    selector: str = "linear"    # "linear": selector network; "softmax": threshold on the top class probability;
                                # "hidden": selector network with one hidden layer of sel_hidden units
    predictor: str = "gap_mlp"  # "gap_mlp": global pool -> FC -> ReLU -> FC; "pool_fc": the paper's Pool(h);
                                # "fc_mlp": the paper's FC(h) on the flattened activation
    in_hw: tuple = (0, 0)       # pool_fc: input map (in_h, in_w), S = in_h*in_w
    out_hw: tuple = (0, 0)      # pool_fc: pooled map (out_h, out_w); features F = C*out_h*out_w
    sel_hidden: int = 0         # selector "hidden": units in the selector's hidden layer
    conv_ks: tuple = (0, 0)     # predictor "conv_fc" (the paper's Conv(k,s)): kernel size, stride; H filters

    @property
    def F(self) -> int:
        if self.predictor == "pool_fc":
            return self.C * self.out_hw[0] * self.out_hw[1]
        if self.predictor == "conv_fc":
            k, s = self.conv_ks
            return self.H * ((self.in_hw[0] - k) // s + 1) * ((self.in_hw[1] - k) // s + 1)
        return self.H if self.predictor == "fc_mlp" else self.C

    def _c(self) -> _Desc:
        return _Desc(self.C, self.S, self.H, self.K, BF16 if self.dtype == "bf16" else F32,
                     NSC if self.layout == "nsc" else NCS, 1 if self.round_operands else 0,
                     float(self.threshold), {"linear": 0, "softmax": 1, "hidden": 2}[self.selector],
                     {"gap_mlp": 0, "pool_fc": 1, "fc_mlp": 2, "conv_fc": 3}[self.predictor], int(self.in_hw[0]), int(self.in_hw[1]),
                     int(self.out_hw[0]), int(self.out_hw[1]), int(self.sel_hidden),
                     int(self.conv_ks[0]), int(self.conv_ks[1]))


def _weights_c(w: dict, keep: list) -> _Weights:
    arrs = {}
    for k in ("W1", "b1", "W2", "b2", "ws", "Ws", "cs", "vs"):
        v = w.get(k)
        arrs[k] = np.ascontiguousarray(v if v is not None else np.zeros(1), dtype=np.float32)
        keep.append(arrs[k])
    return _Weights(_ptr(arrs["W1"]), _ptr(arrs["b1"]), _ptr(arrs["W2"]), _ptr(arrs["b2"]),
                    _ptr(arrs["ws"]), float(w["bs"]), _ptr(arrs["Ws"]), _ptr(arrs["cs"]), _ptr(arrs["vs"]))


def _check_act(d: CacheDef, act: np.ndarray):
    # Both map predictors take either storage order: position s = y*in_w + x of channel c is element
    # [c][s] of a channel-major row and [s][c] of a channels-last row; the features are the same.
    if d.predictor == "pool_fc":
        if d.in_hw[0] * d.in_hw[1] != d.S or min(d.out_hw) < 1 or \
                d.out_hw[0] > d.in_hw[0] or d.out_hw[1] > d.in_hw[1]:
            raise ValueError("pool_fc needs S = in_h*in_w and 1 <= out <= in")
    if d.predictor == "conv_fc":
        k, s = d.conv_ks
        if d.in_hw[0] * d.in_hw[1] != d.S or k < 1 or s < 1 or k > min(d.in_hw):
            raise ValueError("conv_fc needs S = in_h*in_w and 1 <= k <= min(in_h, in_w), s >= 1")
    want = np.uint16 if d.dtype == "bf16" else np.float32
    if act.dtype != want:
        raise TypeError(f"activation dtype {act.dtype}, cache wants {want}")
    if not act.flags["C_CONTIGUOUS"]:
        raise ValueError("activation must be C-contiguous")
    if act.size % (d.C * d.S) != 0:
        raise ValueError("activation size is not a whole number of rows")


def round_bf16(x: float) -> float:
    return float(_load().oracle_round_bf16(float(x)))


def lookup(d: CacheDef, w: dict, act: np.ndarray, row_index: Optional[np.ndarray] = None,
           n: Optional[int] = None) -> dict:
    """Look up n rows.  Returns pooled, logits, probs, pred_class, score, confidence, hit."""
    lib = _load()
    _check_act(d, act)
    rows_avail = act.size // (d.C * d.S)
    if row_index is not None:
        row_index = np.ascontiguousarray(row_index, dtype=np.int32)
        n = len(row_index) if n is None else n
        if n > len(row_index):
            raise ValueError("n exceeds row_index length")
        if n and (row_index[:n].min() < 0 or row_index[:n].max() >= rows_avail):
            raise IndexError("row_index out of range")
    else:
        n = rows_avail if n is None else n
        if n > rows_avail:
            raise ValueError("n exceeds rows in activation")
    out = {
        "pooled": np.zeros((n, d.F), np.float32),
        "logits": np.zeros((n, d.K), np.float32),
        "probs": np.zeros((n, d.K), np.float64),
        "pred_class": np.zeros(n, np.int32),
        "score": np.zeros(n, np.float64),
        "confidence": np.zeros(n, np.float32),
        "hit": np.zeros(n, np.uint8),
    }
    keep: list = []
    dc, wc = d._c(), _weights_c(w, keep)
    rc = lib.oracle_lookup(C.byref(dc), C.byref(wc), _ptr(act), _ptr(row_index), n,
                           _ptr(out["pooled"]), _ptr(out["logits"]), _ptr(out["probs"]),
                           _ptr(out["pred_class"]), _ptr(out["score"]), _ptr(out["confidence"]),
                           _ptr(out["hit"]))
    if rc != 0:
        raise MemoryError("oracle_lookup failed")
    return out


def compact_misses(hit: np.ndarray, ids_in: Optional[np.ndarray] = None) -> np.ndarray:
    lib = _load()
    hit = np.ascontiguousarray(hit, dtype=np.uint8)
    n = len(hit)
    if ids_in is not None:
        ids_in = np.ascontiguousarray(ids_in, dtype=np.int32)
        if len(ids_in) < n:
            raise ValueError("ids_in shorter than hit")
    ids_out = np.zeros(max(n, 1), np.int32)
    m = lib.oracle_compact_misses(_ptr(hit), _ptr(ids_in), n, _ptr(ids_out))
    return ids_out[:m].copy()


# -- step-level access for the pin tests ------------------------------------------------

def pool(d: CacheDef, act: np.ndarray, rows=None) -> np.ndarray:
    lib = _load()
    _check_act(d, act)
    rows = range(act.size // (d.C * d.S)) if rows is None else rows
    dc = d._c()
    out = np.zeros((len(rows), d.F), np.float32)
    fn = lib.oracle_pool_adaptive_row if d.predictor == "pool_fc" else lib.oracle_pool_row
    for i, r in enumerate(rows):
        fn(C.byref(dc), _ptr(act), int(r), _ptr(out[i]))
    return out


def fc1_relu(d: CacheDef, w: dict, p: np.ndarray) -> np.ndarray:
    lib = _load()
    keep: list = []
    dc, wc = d._c(), _weights_c(w, keep)
    p = np.ascontiguousarray(p, np.float32)
    h = np.zeros(d.H, np.float64)
    lib.oracle_fc1_relu(C.byref(dc), C.byref(wc), _ptr(p), _ptr(h))
    return h


def fc2(d: CacheDef, w: dict, h: np.ndarray) -> np.ndarray:
    lib = _load()
    keep: list = []
    dc, wc = d._c(), _weights_c(w, keep)
    h = np.ascontiguousarray(h, np.float64)
    z = np.zeros(d.K, np.float64)
    lib.oracle_fc2(C.byref(dc), C.byref(wc), _ptr(h), _ptr(z))
    return z


def softmax_argmax(z: np.ndarray):
    lib = _load()
    z = np.ascontiguousarray(z, np.float64)
    q = np.zeros_like(z)
    cls = lib.oracle_softmax_argmax(len(z), _ptr(z), _ptr(q))
    return q, int(cls)


def selector_score(d: CacheDef, w: dict, p: np.ndarray, q: np.ndarray) -> float:
    lib = _load()
    keep: list = []
    dc, wc = d._c(), _weights_c(w, keep)
    p = np.ascontiguousarray(p, np.float32)
    q = np.ascontiguousarray(q, np.float64)
    return float(lib.oracle_selector_score(C.byref(dc), C.byref(wc), _ptr(p), _ptr(q)))


def selector_hidden_score(d: CacheDef, w: dict, p: np.ndarray, q: np.ndarray) -> float:
    lib = _load()
    keep: list = []
    dc, wc = d._c(), _weights_c(w, keep)
    p = np.ascontiguousarray(p, np.float32)
    q = np.ascontiguousarray(q, np.float64)
    return float(lib.oracle_selector_hidden_score(C.byref(dc), C.byref(wc), _ptr(p), _ptr(q)))


# -- a stack of caches: layer l+1 looks up only layer l's misses -------------------------

@dataclass
class LayerResult:
    ids_in: np.ndarray      # request ids looked up at this layer, in order
    out: dict               # lookup outputs, row i belongs to ids_in[i]
    ids_out: np.ndarray     # misses that continue


def stack(defs: List[CacheDef], weights: List[dict], acts: List[np.ndarray], batch: int,
          storage: str = "gather") -> List[LayerResult]:
    """Run a whole stack.  storage "gather": acts[l] holds every request, rows are
    indexed by request id.  storage "dense": acts[l] holds only the rows still active,
    row i belonging to the i-th entry of the incoming miss list.
    (Appendix A.1: a hit at an earlier cache removes the sample from later ones.)"""
    ids = np.arange(batch, dtype=np.int32)
    res = []
    for d, w, a in zip(defs, weights, acts):
        if storage == "gather":
            out = lookup(d, w, a, row_index=ids, n=len(ids))
        else:
            out = lookup(d, w, a, row_index=None, n=len(ids))
        ids_out = compact_misses(out["hit"], ids)
        res.append(LayerResult(ids_in=ids, out=out, ids_out=ids_out))
        ids = ids_out
    return res
