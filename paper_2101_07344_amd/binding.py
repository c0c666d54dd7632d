"""ctypes binding with the same names as include/gati.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgati.so")

GATI_OK, GATI_ERR_INVALID_ARG, GATI_ERR_UNSUPPORTED, GATI_ERR_OOM, GATI_ERR_DEVICE = range(5)
GATI_F32, GATI_BF16 = 0, 1
GATI_LAYOUT_NCS, GATI_LAYOUT_NSC = 0, 1
GATI_SEL_LINEAR, GATI_SEL_SOFTMAX, GATI_SEL_HIDDEN = 0, 1, 2
GATI_PRED_GAP_MLP, GATI_PRED_POOL_FC, GATI_PRED_FC_MLP, GATI_PRED_CONV_FC = 0, 1, 2, 3
GATI_COMPACT_STATIC_MAX_ROWS = 1 << 22

# every extern "C" symbol include/gati.h declares
exported_symbols = (
    "gati_cache_create", "gati_cache_destroy", "gati_cache_set_weights", "gati_cache_set_selector", "gati_cache_lookup",
    "gati_cache_lookup_compact", "gati_cache_pool", "gati_compact_misses", "gati_compact_misses_static", "gati_status_string", "gati_cache_pool_variant",
    "gati_trainer_create", "gati_trainer_destroy", "gati_trainer_step", "gati_trainer_get_weights",
    "gati_trainer_get_hidden_selector", "gati_cache_load_trainer", "gati_cache_fork",
    "gati_probe_launch_chain", "gati_probe_stream_read", "gati_probe_copy",
)


class CacheDesc(C.Structure):
    _fields_ = [("C", C.c_int32), ("S", C.c_int32), ("H", C.c_int32), ("K", C.c_int32),
                ("act_dtype", C.c_int), ("layout", C.c_int), ("threshold", C.c_float),
                ("max_rows", C.c_int32), ("selector", C.c_int), ("predictor", C.c_int),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("out_h", C.c_int32), ("out_w", C.c_int32),
                ("selector_hidden", C.c_int32), ("conv_k", C.c_int32), ("conv_s", C.c_int32)]


class CacheWeights(C.Structure):
    _fields_ = [("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
                ("ws", C.c_void_p), ("bs", C.c_float),
                ("Ws", C.c_void_p), ("cs", C.c_void_p), ("vs", C.c_void_p)]


class TrainParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("alpha", C.c_float), ("fp_weight", C.c_float)]


class GatiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {gati_status_string(status)} (status {status})")


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libgati.so (built in-tree by ``python -m paper_2101_07344_amd.build``).
    Raises if it is not there: there is no other implementation to fall back to."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2101_07344_amd.build`")
    try:
        import torch  # noqa: F401  (brings in the HIP runtime the library shares with the caller)
    except Exception:
        pass
    lib = C.CDLL(_LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int32
    lib.gati_cache_create.restype = C.c_int
    lib.gati_cache_create.argtypes = [C.POINTER(CacheDesc), C.POINTER(CacheWeights), C.POINTER(vp)]
    lib.gati_cache_destroy.restype = C.c_int
    lib.gati_cache_destroy.argtypes = [vp]
    lib.gati_cache_set_weights.restype = C.c_int
    lib.gati_cache_set_weights.argtypes = [vp, C.POINTER(CacheWeights)]
    lib.gati_cache_set_selector.restype = C.c_int
    lib.gati_cache_set_selector.argtypes = [vp, C.c_float, C.c_float]
    lib.gati_cache_lookup.restype = C.c_int
    lib.gati_cache_lookup.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.gati_cache_lookup_compact.restype = C.c_int
    lib.gati_cache_lookup_compact.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.gati_cache_pool.restype = C.c_int
    lib.gati_cache_pool.argtypes = [vp, vp, vp, i32, vp, vp, vp]
    lib.gati_compact_misses.restype = C.c_int
    lib.gati_compact_misses.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp]
    lib.gati_compact_misses_static.restype = C.c_int
    lib.gati_compact_misses_static.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp]
    lib.gati_status_string.restype = C.c_char_p
    lib.gati_status_string.argtypes = [C.c_int]
    lib.gati_cache_pool_variant.restype = C.c_char_p
    lib.gati_cache_pool_variant.argtypes = [vp]
    lib.gati_trainer_create.restype = C.c_int
    lib.gati_trainer_create.argtypes = [C.POINTER(CacheDesc), C.POINTER(CacheWeights), C.POINTER(vp)]
    lib.gati_trainer_destroy.restype = C.c_int
    lib.gati_trainer_destroy.argtypes = [vp]
    lib.gati_trainer_step.restype = C.c_int
    lib.gati_trainer_step.argtypes = [vp, vp, i32, i32, vp, vp, i32, C.POINTER(TrainParams), vp, vp]
    lib.gati_trainer_get_weights.restype = C.c_int
    lib.gati_trainer_get_weights.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.gati_trainer_get_hidden_selector.restype = C.c_int
    lib.gati_trainer_get_hidden_selector.argtypes = [vp, vp, vp, vp]
    lib.gati_cache_fork.restype = C.c_int
    lib.gati_cache_fork.argtypes = [vp, C.POINTER(vp)]
    lib.gati_cache_load_trainer.restype = C.c_int
    lib.gati_cache_load_trainer.argtypes = [vp, vp, vp]
    lib.gati_probe_launch_chain.restype = C.c_int
    lib.gati_probe_launch_chain.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp]
    lib.gati_probe_stream_read.restype = C.c_int
    lib.gati_probe_stream_read.argtypes = [vp, C.c_size_t, vp, i32, vp]
    lib.gati_probe_copy.restype = C.c_int
    lib.gati_probe_copy.argtypes = [vp, vp, C.c_size_t, vp]
    _lib = lib
    return lib


def _dptr(t) -> Optional[int]:
    """Device (or host) address of a tensor / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        if not torch.cuda.is_available():
            return None
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ---- the C entry points, one to one ---------------------------------------------------

def gati_status_string(status: int) -> str:
    return load_library().gati_status_string(int(status)).decode()


def gati_cache_create(desc: CacheDesc, weights: CacheWeights):
    """Returns (status, handle)."""
    h = C.c_void_p()
    st = load_library().gati_cache_create(C.byref(desc) if desc is not None else None,
                                          C.byref(weights) if weights is not None else None,
                                          C.byref(h))
    return st, h.value


def gati_cache_destroy(handle) -> int:
    return load_library().gati_cache_destroy(handle)


def gati_cache_set_weights(handle, weights: CacheWeights) -> int:
    return load_library().gati_cache_set_weights(handle, C.byref(weights))


def gati_cache_set_selector(handle, bs: float, threshold: float) -> int:
    return load_library().gati_cache_set_selector(handle, bs, threshold)


def gati_cache_lookup(handle, act, row_index, n_max: int, n_dev, pred_class, confidence, hit,
                      logits=None, stream=None) -> int:
    return load_library().gati_cache_lookup(handle, _dptr(act), _dptr(row_index), int(n_max), _dptr(n_dev),
                                            _dptr(pred_class), _dptr(confidence), _dptr(hit),
                                            _dptr(logits), _stream(stream))


def gati_cache_lookup_compact(handle, act, row_index, n_max: int, n_dev, pred_class, confidence, hit,
                              logits, ids_in, ids_out, n_miss_dev, stream=None) -> int:
    return load_library().gati_cache_lookup_compact(
        handle, _dptr(act), _dptr(row_index), int(n_max), _dptr(n_dev), _dptr(pred_class), _dptr(confidence),
        _dptr(hit), _dptr(logits), _dptr(ids_in), _dptr(ids_out), _dptr(n_miss_dev), _stream(stream))


def gati_cache_pool(handle, act, row_index, n_max: int, n_dev, pooled, stream=None) -> int:
    return load_library().gati_cache_pool(handle, _dptr(act), _dptr(row_index), int(n_max), _dptr(n_dev),
                                          _dptr(pooled), _stream(stream))


def gati_compact_misses(handle, hit, ids_in, n_max: int, n_dev, ids_out, n_miss_dev, stream=None) -> int:
    return load_library().gati_compact_misses(handle, _dptr(hit), _dptr(ids_in), int(n_max), _dptr(n_dev),
                                              _dptr(ids_out), _dptr(n_miss_dev), _stream(stream))


def gati_compact_misses_static(handle, hit, ids_in, n_max: int, n_dev, ids_out, n_miss_dev, stream=None) -> int:
    return load_library().gati_compact_misses_static(handle, _dptr(hit), _dptr(ids_in), int(n_max), _dptr(n_dev),
                                                     _dptr(ids_out), _dptr(n_miss_dev), _stream(stream))


def gati_probe_stream_read(buf, nbytes: int, sink, blocks_per_cu: int = 1, stream=None) -> int:
    return load_library().gati_probe_stream_read(_dptr(buf), int(nbytes), _dptr(sink), int(blocks_per_cu), _stream(stream))


def gati_probe_launch_chain(cell, links: int, workgroups: int, loads: int, stream=None) -> int:
    return load_library().gati_probe_launch_chain(_dptr(cell), int(links), int(workgroups), int(loads), _stream(stream))


def gati_probe_copy(dst, src, nbytes: int, stream=None) -> int:
    return load_library().gati_probe_copy(_dptr(dst), _dptr(src), int(nbytes), _stream(stream))


def gati_cache_pool_variant(handle) -> str:
    return load_library().gati_cache_pool_variant(handle).decode()


# ---- small conveniences over the handles (still marshalling only) -----------------------

def _check(st: int, where: str):
    if st != GATI_OK:
        raise GatiError(st, where)


class Cache:
    """Owns one gati_cache_t."""

    def __init__(self, C_: int, S: int, H: int, K: int, dtype: str, layout: str, threshold: float,
                 max_rows: int, weights: dict, selector: str = "linear", predictor: str = "gap_mlp",
                 in_hw=(0, 0), out_hw=(0, 0), sel_hidden: int = 0, conv_ks=(0, 0)):
        self.C, self.S, self.H, self.K = C_, S, H, K
        self.dtype, self.layout, self.max_rows = dtype, layout, max_rows
        self.threshold = float(threshold)
        pool_fc, fc_mlp, conv_fc = predictor == "pool_fc", predictor == "fc_mlp", predictor == "conv_fc"
        # features per row that the selector sees and gati_cache_pool reports
        self.F = C_ * out_hw[0] * out_hw[1] if pool_fc else (H if fc_mlp else C_)
        if conv_fc:
            k, s = conv_ks
            self.F = H * ((in_hw[0] - k) // s + 1) * ((in_hw[1] - k) // s + 1)
        desc = CacheDesc(C_, S, 0 if pool_fc else H, K, GATI_BF16 if dtype == "bf16" else GATI_F32,
                         GATI_LAYOUT_NSC if layout == "nsc" else GATI_LAYOUT_NCS, float(threshold), max_rows,
                         {"linear": GATI_SEL_LINEAR, "softmax": GATI_SEL_SOFTMAX, "hidden": GATI_SEL_HIDDEN}[selector],
                         {"gap_mlp": GATI_PRED_GAP_MLP, "pool_fc": GATI_PRED_POOL_FC, "fc_mlp": GATI_PRED_FC_MLP,
                          "conv_fc": GATI_PRED_CONV_FC}[predictor],
                         int(in_hw[0]), int(in_hw[1]), int(out_hw[0]), int(out_hw[1]), int(sel_hidden),
                         int(conv_ks[0]), int(conv_ks[1]))
        self._shape = (C_, S, H, K, pool_fc, fc_mlp, conv_fc, selector == "hidden", sel_hidden, tuple(conv_ks))
        self._softmax_sel = selector == "softmax"
        w, _keep = self._marshal(weights)
        st, self.handle = gati_cache_create(desc, w)
        _check(st, "gati_cache_create")

    @classmethod
    def from_layer(cls, L, weights: dict, max_rows: int) -> "Cache":
        """Build from any record with the fields C, S, H, K, dtype, layout, threshold and,
        optionally, predictor, in_hw, out_hw, selector, sel_hidden."""
        return cls(L.C, L.S, L.H, L.K, L.dtype, L.layout, L.threshold, max_rows, weights,
                   selector=getattr(L, "selector", "linear"), predictor=getattr(L, "predictor", "gap_mlp"),
                   in_hw=getattr(L, "in_hw", (0, 0)), out_hw=getattr(L, "out_hw", (0, 0)),
                   sel_hidden=getattr(L, "sel_hidden", 0), conv_ks=getattr(L, "conv_ks", (0, 0)))

    def _marshal(self, weights: dict):
        """Host fp32 arrays of the shapes this cache was created with -> the C struct (and the
        arrays it points into, which must outlive the call)."""
        C_, S, H, K, pool_fc, fc_mlp, conv_fc, hidden_sel, sel_hidden, conv_ks = self._shape
        names = ("W2", "b2") if pool_fc else ("W1", "b1", "W2", "b2")
        names += ("Ws", "cs", "vs") if hidden_sel else ("ws",)
        if "ws" in names and weights.get("ws") is None and self._softmax_sel:
            names = tuple(k for k in names if k != "ws")     # the softmax-threshold mode reads no selector weights
        keep = {k: np.ascontiguousarray(weights[k], dtype=np.float32) for k in names}
        if conv_fc:
            assert keep["W1"].shape == (H, C_, conv_ks[0], conv_ks[0])
        elif not pool_fc:
            assert keep["W1"].shape == (H, C_ * S if fc_mlp else C_)
        assert keep["W2"].shape == (K, self.F if (pool_fc or conv_fc) else H)
        if hidden_sel:
            assert keep["Ws"].shape == (sel_hidden, self.F + K) and keep["cs"].shape == (sel_hidden,) \
                and keep["vs"].shape == (sel_hidden,)
        elif "ws" in keep:
            assert keep["ws"].shape == (self.F + K,)
        ptr = lambda k: keep[k].ctypes.data if k in keep else None
        w = CacheWeights(ptr("W1"), ptr("b1"), ptr("W2"), ptr("b2"), ptr("ws"), float(weights.get("bs", 0.0)),
                         ptr("Ws"), ptr("cs"), ptr("vs"))
        return w, keep

    def set_weights(self, weights: dict):
        w, _keep = self._marshal(weights)
        _check(gati_cache_set_weights(self.handle, w), "gati_cache_set_weights")

    def fork(self) -> "Cache":
        """A handle with its own workspace on the same weights, for lookups that overlap in time with this one's."""
        import copy
        st, handle = gati_cache_fork(self.handle)
        _check(st, "gati_cache_fork")
        other = copy.copy(self)
        other.handle = handle
        return other

    def load_trainer(self, trainer: "Trainer", stream=None):
        _check(gati_cache_load_trainer(self.handle, trainer.handle, stream), "gati_cache_load_trainer")

    def lookup(self, act, row_index, n_max, n_dev, pred_class, confidence, hit, logits=None, stream=None):
        _check(gati_cache_lookup(self.handle, act, row_index, n_max, n_dev, pred_class, confidence, hit,
                                 logits, stream), "gati_cache_lookup")

    def lookup_compact(self, act, row_index, n_max, n_dev, pred_class, confidence, hit, logits,
                       ids_in, ids_out, n_miss_dev, stream=None):
        _check(gati_cache_lookup_compact(self.handle, act, row_index, n_max, n_dev, pred_class, confidence,
                                         hit, logits, ids_in, ids_out, n_miss_dev, stream),
               "gati_cache_lookup_compact")

    def pool(self, act, row_index, n_max, n_dev, pooled, stream=None):
        _check(gati_cache_pool(self.handle, act, row_index, n_max, n_dev, pooled, stream), "gati_cache_pool")

    def compact(self, hit, ids_in, n_max, n_dev, ids_out, n_miss_dev, stream=None):
        _check(gati_compact_misses(self.handle, hit, ids_in, n_max, n_dev, ids_out, n_miss_dev, stream),
               "gati_compact_misses")

    def set_selector(self, bs: float, threshold: float):
        _check(gati_cache_set_selector(self.handle, bs, threshold), "gati_cache_set_selector")
        self.threshold = float(threshold)

    @property
    def pool_variant(self) -> str:
        return gati_cache_pool_variant(self.handle)

    def close(self):
        if getattr(self, "handle", None):
            gati_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gati_trainer_create(desc: CacheDesc, weights: CacheWeights):
    """Returns (status, handle)."""
    h = C.c_void_p()
    st = load_library().gati_trainer_create(C.byref(desc) if desc is not None else None,
                                            C.byref(weights) if weights is not None else None, C.byref(h))
    return st, h.value


def gati_trainer_destroy(handle) -> int:
    return load_library().gati_trainer_destroy(handle)


def gati_trainer_step(handle, pooled, ld_pooled, n, labels, teacher, ld_teacher, params, losses=None, stream=None) -> int:
    return load_library().gati_trainer_step(handle, _dptr(pooled), ld_pooled, n, _dptr(labels), _dptr(teacher),
                                            ld_teacher, C.byref(params) if params is not None else None,
                                            _dptr(losses), _stream(stream))


def gati_trainer_get_weights(handle, W1, b1, W2, b2, ws, bs) -> int:
    """Host numpy fp32 arrays (bs: a 1-element array) filled in place."""
    a = lambda x: x.ctypes.data if x is not None else None
    return load_library().gati_trainer_get_weights(handle, a(W1), a(b1), a(W2), a(b2), a(ws), a(bs))


def gati_cache_fork(cache_handle):
    out = C.c_void_p()
    st = load_library().gati_cache_fork(cache_handle, C.byref(out))
    return st, out.value


def gati_cache_load_trainer(cache_handle, trainer_handle, stream=None) -> int:
    return load_library().gati_cache_load_trainer(cache_handle, trainer_handle, _stream(stream))


def gati_trainer_get_hidden_selector(handle, Ws, cs, vs) -> int:
    a = lambda x: x.ctypes.data if x is not None else None
    return load_library().gati_trainer_get_hidden_selector(handle, a(Ws), a(cs), a(vs))


class Trainer:
    """SGD steps on one cache's predictor and selector.  predictor: "gap_mlp" (input rows = pooled features
    [n, C]), "pool_fc" (the paper's Pool(h): input rows = the C*out_h*out_w window means, no hidden layer, H
    ignored), "fc_mlp" (the paper's FC(h): input rows = the flattened activation [n, C*S] as fp32) or "conv_fc"
    (the paper's Conv(k,s): input rows = the channel-major map [n, C*in_h*in_w] as fp32, H filters).
    selector: "linear", "hidden" (sel_hidden > 0 units; weights hold Ws, cs, vs) or "softmax" (no selector
    network: the predictor alone is trained)."""

    def __init__(self, C_: int, H: int, K: int, weights: dict, max_rows: int, sel_hidden: int = 0,
                 predictor: str = "gap_mlp", out_hw=(0, 0), S: int = 1, in_hw=(0, 0), conv_ks=(0, 0), selector: str = None):
        pool_fc, fc_mlp, conv_fc = predictor == "pool_fc", predictor == "fc_mlp", predictor == "conv_fc"
        assert predictor in ("gap_mlp", "pool_fc", "fc_mlp", "conv_fc")
        selector = selector or ("hidden" if sel_hidden else "linear")
        sel_hidden = int(sel_hidden) if selector == "hidden" else 0
        H = 0 if pool_fc else H
        if conv_fc:
            S = in_hw[0] * in_hw[1]
            k, s = conv_ks
            P = ((in_hw[0] - k) // s + 1) * ((in_hw[1] - k) // s + 1)
        # width of the input rows, inputs of the output layer, features the selector reads
        Cin = C_ * out_hw[0] * out_hw[1] if pool_fc else (C_ * S if (fc_mlp or conv_fc) else C_)
        Hin = Cin if pool_fc else (H * P if conv_fc else H)
        Fsel = Hin if (fc_mlp or conv_fc) else Cin
        names = ("W2", "b2") if pool_fc else ("W1", "b1", "W2", "b2")
        names += {"hidden": ("Ws", "cs", "vs"), "linear": ("ws",), "softmax": ()}[selector]
        keep = {k: np.ascontiguousarray(weights[k], dtype=np.float32) for k in names}
        if conv_fc:
            assert keep["W1"].shape == (H, C_, conv_ks[0], conv_ks[0]) and keep["b1"].shape == (H,)
        elif not pool_fc:
            assert keep["W1"].shape == (H, Cin) and keep["b1"].shape == (H,)
        assert keep["W2"].shape == (K, Hin) and keep["b2"].shape == (K,)
        if selector == "hidden":
            assert keep["Ws"].shape == (sel_hidden, Fsel + K) and keep["cs"].shape == (sel_hidden,) \
                and keep["vs"].shape == (sel_hidden,)
        elif selector == "linear":
            assert keep["ws"].shape == (Fsel + K,)
        desc = CacheDesc(C_, S, H, K, GATI_F32, GATI_LAYOUT_NCS, 0.5, max_rows,
                         {"linear": GATI_SEL_LINEAR, "hidden": GATI_SEL_HIDDEN, "softmax": GATI_SEL_SOFTMAX}[selector],
                         {"gap_mlp": GATI_PRED_GAP_MLP, "pool_fc": GATI_PRED_POOL_FC, "fc_mlp": GATI_PRED_FC_MLP,
                          "conv_fc": GATI_PRED_CONV_FC}[predictor],
                         int(in_hw[0]), int(in_hw[1]), int(out_hw[0]), int(out_hw[1]), sel_hidden,
                         int(conv_ks[0]), int(conv_ks[1]))
        ptr = lambda k: keep[k].ctypes.data if k in keep else None
        w = CacheWeights(ptr("W1"), ptr("b1"), ptr("W2"), ptr("b2"), ptr("ws"), float(weights.get("bs", 0.0)),
                         ptr("Ws"), ptr("cs"), ptr("vs"))
        st, self.handle = gati_trainer_create(desc, w)
        _check(st, "gati_trainer_create")
        self.C, self.H, self.K, self.max_rows, self.sel_hidden = Cin, H, K, max_rows, sel_hidden
        self.Hin, self.Fsel, self.selector = Hin, Fsel, selector
        self._w1_shape = (H, C_, conv_ks[0], conv_ks[0]) if conv_fc else (H, Cin)

    def step(self, pooled, labels, teacher, lr: float, alpha: float, fp_weight: float, losses=None, stream=None,
             n: Optional[int] = None):
        """pooled [n, >=C] fp32, labels [n] int32, teacher [n, >=K] fp32: device tensors."""
        n = pooled.shape[0] if n is None else n
        import torch
        assert pooled.dtype == torch.float32 and teacher.dtype == torch.float32 and labels.dtype == torch.int32
        assert pooled.stride(1) == 1 and teacher.stride(1) == 1 and labels.stride(0) == 1
        assert pooled.shape[1] >= self.C and teacher.shape[1] >= self.K and labels.shape[0] >= n
        _check(gati_trainer_step(self.handle, pooled, pooled.stride(0), n, labels, teacher, teacher.stride(0),
                                 TrainParams(lr, alpha, fp_weight), losses, stream), "gati_trainer_step")

    def fit(self, pooled, labels, teacher, epochs: int, batch_size: int, lr: float, alpha: float, fp_weight: float,
            losses=None, stream=None):
        """Mini-batch SGD in storage order: `epochs` sweeps over the samples in batches of `batch_size`
        (the last one may be shorter); the paper retrains for 5 epochs (Section 7).  losses: optional
        device [epochs, batches, 2] tensor receiving every step's two losses.  Only enqueues."""
        n = pooled.shape[0]
        assert 0 < batch_size <= self.max_rows
        for e in range(epochs):
            for b, lo in enumerate(range(0, n, batch_size)):
                hi = min(n, lo + batch_size)
                self.step(pooled[lo:hi], labels[lo:hi], teacher[lo:hi], lr, alpha, fp_weight,
                          None if losses is None else losses[e, b], stream)

    def get_weights(self) -> dict:
        out = {"W2": np.empty((self.K, self.Hin), np.float32), "b2": np.empty(self.K, np.float32)}
        if self.H:
            out.update({"W1": np.empty(self._w1_shape, np.float32), "b1": np.empty(self.H, np.float32)})
        if self.selector == "linear":
            out["ws"] = np.empty(self.Fsel + self.K, np.float32)
        bs = np.empty(1, np.float32)
        _check(gati_trainer_get_weights(self.handle, out.get("W1"), out.get("b1"), out["W2"], out["b2"], out.get("ws"), bs),
               "gati_trainer_get_weights")
        if self.selector != "softmax":
            out["bs"] = float(bs[0])
        if self.selector == "hidden":
            out.update({"Ws": np.empty((self.sel_hidden, self.Fsel + self.K), np.float32),
                        "cs": np.empty(self.sel_hidden, np.float32), "vs": np.empty(self.sel_hidden, np.float32)})
            _check(gati_trainer_get_hidden_selector(self.handle, out["Ws"], out["cs"], out["vs"]),
                   "gati_trainer_get_hidden_selector")
        return out

    def close(self):
        if getattr(self, "handle", None):
            gati_trainer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class CacheStack:
    """A stack of caches with the device buffers one pass needs, chained on the device:
    layer l+1 looks up only layer l's misses, and the miss count never visits the host."""

    def __init__(self, caches: Sequence[Cache], batch: int, storage: str = "gather", keep_logits: bool = False,
                 first_id: int = 0):
        """first_id: request id of this stack's first row (a stack may own a slice of a larger
        batch whose activation tensors are indexed by global request id)."""
        import torch
        self.caches, self.batch, self.storage = list(caches), batch, storage
        dev = "cuda"
        L = len(self.caches)
        self.ids = [torch.empty(batch, dtype=torch.int32, device=dev) for _ in range(L + 1)]
        self.ids[0].copy_(torch.arange(first_id, first_id + batch, dtype=torch.int32))
        self.counts = torch.zeros(L + 1, dtype=torch.int32, device=dev)
        self.counts[0] = batch
        self.pred_class = [torch.zeros(batch, dtype=torch.int32, device=dev) for _ in range(L)]
        self.confidence = [torch.zeros(batch, dtype=torch.float32, device=dev) for _ in range(L)]
        self.hit = [torch.zeros(batch, dtype=torch.uint8, device=dev) for _ in range(L)]
        self.logits = ([torch.zeros(batch, c.K, dtype=torch.float32, device=dev) for c in self.caches]
                       if keep_logits else [None] * L)

    def run(self, acts: Sequence, stream=None, fused: bool = True):
        """Enqueue one pass over all layers.  acts[l] is the layer's activation tensor:
        the full batch indexed by request id ("gather"), or the rows still active in
        miss-list order ("dense").  fused: one gati_cache_lookup_compact per layer instead of
        gati_cache_lookup + gati_compact_misses (same results)."""
        for l in range(len(self.caches)):
            self.run_layer(l, acts[l], stream, fused)

    def run_layer(self, l: int, act, stream=None, fused: bool = True):
        """Enqueue layer l alone (lookup of the rows still active + compaction of its misses)."""
        es = self.counts.element_size()
        cbase = self.counts.data_ptr()
        cache = self.caches[l]
        n_dev = cbase + l * es
        row_index = self.ids[l] if self.storage == "gather" else None
        if fused:
            cache.lookup_compact(act, row_index, self.batch, n_dev, self.pred_class[l],
                                 self.confidence[l], self.hit[l], self.logits[l], self.ids[l],
                                 self.ids[l + 1], cbase + (l + 1) * es, stream)
        else:
            cache.lookup(act, row_index, self.batch, n_dev, self.pred_class[l], self.confidence[l],
                         self.hit[l], self.logits[l], stream)
            cache.compact(self.hit[l], self.ids[l], self.batch, n_dev, self.ids[l + 1],
                          cbase + (l + 1) * es, stream)

    def close(self):
        for c in self.caches:
            c.close()
