"""Thin ctypes binding of libgbt.so.

Argument marshalling only: every step of the path runs inside the library's HIP
kernels.  torch supplies device memory (``tensor.data_ptr()``) and the stream.
There is no fallback: if the library has not been built, or there is no
MI355X, loading or ``Context()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgbt.so")

OK, EINVAL, ENOMEM, EHIP, EUNSUPPORTED = 0, -1, -2, -3, -4
PARTITION_STATIC_MAX_ROWS = 1 << 22   # GBT_PARTITION_STATIC_MAX_ROWS
OBJECTIVES = {"squared": 0, "logistic": 1}

# every symbol include/gbt.h declares
SYMBOLS = [
    "gbt_create", "gbt_destroy", "gbt_last_error", "gbt_version",
    "gbt_quantise_workspace_bytes", "gbt_quantise", "gbt_quantise_packed", "gbt_bits", "gbt_packed_words", "gbt_compress",
    "gbt_gradients", "gbt_gpair_fixed", "gbt_sum_gpair", "gbt_build_hist", "gbt_hist_subtract",
    "gbt_hist_export_f64", "gbt_eval_split", "gbt_partition_workspace_bytes", "gbt_partition",
    "gbt_partition_static",
    "gbt_grow_tree_workspace_bytes", "gbt_grow_tree_path", "gbt_grow_tree",
    "gbt_grow_tree_lossguide_workspace_bytes", "gbt_grow_tree_lossguide", "gbt_boost_round",
    "gbt_predict_workspace_bytes", "gbt_predict",
    "gbt_profile_enable", "gbt_profile_read", "gbt_measure_stream_read",
    "gbt_sparse_entry_bytes", "gbt_sparse_capacity", "gbt_compress_sparse_workspace_bytes", "gbt_compress_sparse_count", "gbt_compress_sparse",
    "gbt_build_hist_sparse", "gbt_grow_tree_sparse_workspace_bytes", "gbt_grow_tree_sparse", "gbt_predict_sparse",
    "gbt_grow_tree_sparse_lossguide_workspace_bytes", "gbt_grow_tree_sparse_lossguide",
]

PROF_LEVELS = 18   # GBT_PROF_LEVELS
PROF_CLASSES = ["hist_root", "hist_node", "partition", "eval", "clear", "other", "hist_first", "hist_inplace"]


class GbtError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"libgbt error {code}: {text}")
        self.code = code


class Params(C.Structure):
    _fields_ = [("max_depth", C.c_int32), ("max_bins", C.c_int32), ("lambda_", C.c_double),
                ("gamma", C.c_double), ("min_child_weight", C.c_double), ("eta", C.c_double),
                ("objective", C.c_int32), ("base_margin", C.c_float)]


class Split(C.Structure):
    _fields_ = [("feature", C.c_int32), ("bin", C.c_int32), ("default_left", C.c_int32),
                ("valid", C.c_int32), ("gain", C.c_double), ("GL", C.c_double), ("HL", C.c_double),
                ("GR", C.c_double), ("HR", C.c_double), ("GLq", C.c_int64), ("HLq", C.c_int64)]


class Profile(C.Structure):
    _fields_ = [("ms", C.c_double * 8), ("bytes", C.c_double * 8), ("launches", C.c_int64 * 8),
                ("alg_bytes", C.c_double * 8), ("level_ms", C.c_double * PROF_LEVELS),
                ("level_alg_bytes", C.c_double * PROF_LEVELS), ("level_row_features", C.c_double * PROF_LEVELS),
                ("level_launches", C.c_int64 * PROF_LEVELS)]


class Tree(C.Structure):
    _fields_ = [("capacity", C.c_int32), ("n_nodes", C.c_int32),
                ("feature", C.c_void_p), ("bin", C.c_void_p), ("default_left", C.c_void_p),
                ("left", C.c_void_p), ("right", C.c_void_p), ("threshold", C.c_void_p),
                ("weight", C.c_void_p), ("gain", C.c_void_p), ("sumG", C.c_void_p),
                ("sumH", C.c_void_p), ("n_rows", C.c_void_p)]


_TREE_FIELDS = [("feature", np.int32), ("bin", np.int32), ("default_left", np.int32), ("left", np.int32),
                ("right", np.int32), ("threshold", np.float32), ("weight", np.float64),
                ("gain", np.float64), ("sumG", np.float64), ("sumH", np.float64), ("n_rows", np.int64)]

_lib = None


def load():
    """Load libgbt.so (built in-tree by ``paper_1806_11248_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1806_11248_amd.build` "
                           "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    L.gbt_version.restype = C.c_char_p
    L.gbt_last_error.restype = C.c_char_p
    L.gbt_last_error.argtypes = [C.c_void_p]
    L.gbt_create.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_void_p]
    L.gbt_destroy.argtypes = [C.c_void_p]
    L.gbt_bits.argtypes = [C.c_uint32]
    L.gbt_packed_words.restype = C.c_int64
    L.gbt_packed_words.argtypes = [C.c_int64, C.c_int32, C.c_int32]
    for nm in ("gbt_quantise_workspace_bytes", "gbt_partition_workspace_bytes",
               "gbt_grow_tree_workspace_bytes", "gbt_predict_workspace_bytes"):
        getattr(L, nm).restype = C.c_size_t
    L.gbt_quantise_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int64, C.c_int32]
    L.gbt_partition_workspace_bytes.argtypes = [C.c_int64]
    L.gbt_grow_tree_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    L.gbt_grow_tree_lossguide_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    L.gbt_grow_tree_lossguide_workspace_bytes.restype = C.c_size_t
    L.gbt_grow_tree_path.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    L.gbt_grow_tree_path.restype = C.c_int32
    L.gbt_predict_workspace_bytes.argtypes = [C.c_void_p, C.c_int32]
    vp, i32, i64, u32, f64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_double, C.c_size_t
    L.gbt_quantise.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, vp, vp, vp, vp, vp, vp, sz]
    L.gbt_compress.argtypes = [vp, vp, i64, i32, u32, vp, vp]
    L.gbt_gradients.argtypes = [vp, i32, vp, vp, i64, vp]
    L.gbt_gpair_fixed.argtypes = [vp, vp, i64, vp, vp, vp, sz]
    L.gbt_sum_gpair.argtypes = [vp, vp, vp, i64, vp, vp, sz]
    L.gbt_build_hist.argtypes = [vp, vp, i32, i64, i32, i32, i32, vp, i64, vp, vp]
    L.gbt_hist_subtract.argtypes = [vp, vp, vp, vp, i64]
    L.gbt_hist_export_f64.argtypes = [vp, vp, i32, i32, vp, vp]
    L.gbt_eval_split.argtypes = [vp, vp, vp, i32, i32, i64, i64, vp, vp, vp, vp, sz]
    L.gbt_partition.argtypes = [vp, vp, i32, i64, i32, vp, i64, i64, i32, i32, i32, i32, vp, sz, vp]
    L.gbt_partition_static.argtypes = [vp, vp, i32, i64, i32, vp, i64, i64, i32, i32, i32, i32, vp]
    L.gbt_grow_tree.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz]
    L.gbt_grow_tree_lossguide.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz]
    L.gbt_boost_round.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz]
    L.gbt_predict.argtypes = [vp, vp, i32, vp, i32, i32, vp, i64, i32, f64, vp, vp, sz]
    L.gbt_sparse_entry_bytes.argtypes = [i32, i32]
    L.gbt_sparse_capacity.argtypes = [i64]
    L.gbt_sparse_capacity.restype = i64
    L.gbt_compress_sparse_workspace_bytes.argtypes = [i64]
    L.gbt_compress_sparse_workspace_bytes.restype = sz
    L.gbt_compress_sparse_count.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp, sz]
    L.gbt_compress_sparse.argtypes = [vp, vp, i64, i32, i32, i32, vp, i64, vp, i64]
    L.gbt_build_hist_sparse.argtypes = [vp, vp, vp, i64, i32, i32, i64, i64, vp, vp]
    L.gbt_grow_tree_sparse_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
    L.gbt_grow_tree_sparse_workspace_bytes.restype = sz
    L.gbt_grow_tree_sparse.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz]
    L.gbt_grow_tree_sparse_lossguide_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
    L.gbt_grow_tree_sparse_lossguide_workspace_bytes.restype = sz
    L.gbt_grow_tree_sparse_lossguide.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz]
    L.gbt_predict_sparse.argtypes = [vp, vp, i32, vp, vp, i64, i32, i32, f64, vp, vp, sz]
    L.gbt_profile_enable.argtypes = [vp, i32]
    L.gbt_profile_read.argtypes = [vp, vp]
    L.gbt_measure_stream_read.argtypes = [vp, vp, sz, i32, vp, vp, sz]
    _lib = L
    return L


def bits_for(max_value: int) -> int:
    return int(load().gbt_bits(max_value))


def packed_words(n: int, F: int, bits: int) -> int:
    return int(load().gbt_packed_words(n, F, bits))


def make_params(*, max_depth, max_bins, lam=1.0, gamma=0.0, min_child_weight=1.0, eta=1.0,
                objective="squared", base_margin=0.0) -> Params:
    return Params(max_depth, max_bins, lam, gamma, min_child_weight, eta,
                  OBJECTIVES.get(objective, 0), base_margin)


def new_tree(max_depth: int) -> dict:
    cap = 2 ** (max_depth + 1) - 1
    t = {nm: np.zeros(cap, dt) for nm, dt in _TREE_FIELDS}
    t["capacity"] = cap
    t["n_nodes"] = 0
    return t


def new_tree_leaves(max_leaves: int) -> dict:
    """Arrays for a tree of at most max_leaves leaves (2*max_leaves - 1 nodes)."""
    cap = max(1, 2 * max_leaves - 1)   # a bad budget is the library's to refuse
    t = {nm: np.zeros(cap, dt) for nm, dt in _TREE_FIELDS}
    t["capacity"] = cap
    t["n_nodes"] = 0
    return t


def _tree_struct(t: dict) -> Tree:
    s = Tree()
    s.capacity = int(t["capacity"])
    s.n_nodes = int(t["n_nodes"])
    for nm, _ in _TREE_FIELDS:
        setattr(s, nm, t[nm].ctypes.data)
    return s


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _need(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of {dtype}")
    return t


class Context:
    """One libgbt context bound to a device and to torch's current stream."""

    def __init__(self, device: int = 0, stream=None):
        self.lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("libgbt needs a GPU: no HIP device is visible")
        self.device = torch.device("cuda", device)
        torch.cuda.set_device(self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        st = self.lib.gbt_create(C.byref(h), device, C.c_void_p(self.stream.cuda_stream))
        if st != OK:
            raise GbtError(st, "gbt_create failed (see stderr)")
        self.h = h
        self._ws = {}

    def close(self):
        if getattr(self, "h", None):
            self.lib.gbt_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers -----------------------------------------------------------
    def _check(self, st):
        if st != OK:
            raise GbtError(st, self.lib.gbt_last_error(self.h).decode())

    def workspace(self, key: str, nbytes: int) -> torch.Tensor:
        """A cached byte buffer of at least nbytes (device memory comes from torch)."""
        w = self._ws.get(key)
        if w is None or w.numel() < nbytes:
            self._ws.pop(key, None)
            w = torch.empty(max(int(nbytes), 4096), dtype=torch.uint8, device=self.device)
            self._ws[key] = w
        return w

    def empty(self, shape, dtype):
        return torch.empty(shape, dtype=dtype, device=self.device)

    # -- measurement -----------------------------------------------------------
    def profile_enable(self, on: bool = True):
        self._check(self.lib.gbt_profile_enable(self.h, int(on)))

    def profile_read(self) -> dict:
        p = Profile()
        self._check(self.lib.gbt_profile_read(self.h, C.byref(p)))
        out = {nm: dict(ms=p.ms[i], bytes=p.bytes[i], alg_bytes=p.alg_bytes[i], launches=p.launches[i])
               for i, nm in enumerate(PROF_CLASSES)}
        self.last_profile_levels = [dict(level=k, ms=p.level_ms[k], alg_bytes=p.level_alg_bytes[k],
                                         row_features=p.level_row_features[k], launches=p.level_launches[k])
                                    for k in range(PROF_LEVELS) if p.level_launches[k]]
        return out

    def measure_stream_read(self, buf, reps: int = 5) -> float:
        """GB/s of a kernel that only reads `buf` (a device tensor), best of `reps` launches."""
        ws = self.workspace("small", 4096)
        out = C.c_double()
        self._check(self.lib.gbt_measure_stream_read(self.h, _ptr(buf), buf.numel() * buf.element_size(), reps,
                                                     C.byref(out), _ptr(ws), ws.numel()))
        return out.value

    # -- Sec. 2.1 ------------------------------------------------------------
    def quantise(self, X=None, csr=None, *, max_bins: int, n=None, F=None):
        """Returns (cuts [F][max_bins-1], nb [F], sym uint16 [n][F], max_value, missing_sym)."""
        if X is not None:
            _need(X, torch.float32, "X")
            n, F = X.shape
            n_values = n * F
            args = (_ptr(X), None, None, None)
        else:
            indptr, indices, values = csr
            _need(indptr, torch.int64, "indptr"); _need(indices, torch.int32, "indices")
            _need(values, torch.float32, "values")
            n_values = values.numel()
            args = (None, _ptr(indptr), _ptr(indices), _ptr(values))
        cuts = self.empty((F, max_bins - 1), torch.float32)
        nb = self.empty((F,), torch.int32)
        sym = self.empty((n, F), torch.uint16)
        ws_bytes = self.lib.gbt_quantise_workspace_bytes(n, F, n_values, max_bins)
        ws = self.workspace("quantise", ws_bytes)
        mv, ms = C.c_int32(), C.c_int32()
        self._check(self.lib.gbt_quantise(self.h, *args, n, F, max_bins, _ptr(cuts), _ptr(nb), _ptr(sym),
                                          C.byref(mv), C.byref(ms), _ptr(ws), ws.numel()))
        self._ws.pop("quantise", None)   # large and used once
        return cuts, nb, sym, mv.value, ms.value

    def quantise_packed(self, X=None, csr=None, *, max_bins: int, n=None, F=None):
        """Cuts and the packed matrix in one call (no symbol matrix in between).
        Returns (cuts [F][max_bins-1], nb [F], packed int32 words, bits, max_value, missing_sym)."""
        if X is not None:
            _need(X, torch.float32, "X")
            n, F = X.shape
            n_values = n * F
            args = (_ptr(X), None, None, None)
        else:
            indptr, indices, values = csr
            _need(indptr, torch.int64, "indptr"); _need(indices, torch.int32, "indices")
            _need(values, torch.float32, "values")
            n_values = values.numel()
            args = (None, _ptr(indptr), _ptr(indices), _ptr(values))
        cuts = self.empty((F, max_bins - 1), torch.float32)
        nb = self.empty((F,), torch.int32)
        cap = packed_words(n, F, bits_for(max_bins))      # no symbol exceeds max_bins
        packed = self.empty((cap,), torch.int32)
        ws_bytes = self.lib.gbt_quantise_workspace_bytes(n, F, n_values, max_bins)
        ws = self.workspace("quantise", ws_bytes)
        mv, ms, b = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(self.lib.gbt_quantise_packed(self.h, *args, n, F, max_bins, _ptr(cuts), _ptr(nb), _ptr(packed),
                                                 C.c_int64(cap), C.byref(b), C.byref(mv), C.byref(ms), _ptr(ws),
                                                 ws.numel()))
        self._ws.pop("quantise", None)   # large and used once
        return cuts, nb, packed[:packed_words(n, F, b.value)], b.value, mv.value, ms.value

    # -- Sec. 2.2 ------------------------------------------------------------
    def compress(self, sym, max_value: int):
        _need(sym, torch.uint16, "sym")
        n, F = sym.shape
        bits = bits_for(max_value)
        packed = self.empty((packed_words(n, F, bits),), torch.int32)
        b = C.c_int32()
        self._check(self.lib.gbt_compress(self.h, _ptr(sym), n, F, max_value, _ptr(packed), C.byref(b)))
        return packed, b.value

    def compress_sparse(self, sym, max_bins: int, missing_sym: int):
        """Sparse rows of sym[n][F]: (rowptr uint32[n+1] as int32 tensor, ent[capacity], nnz); the entries are
        uint16 where F * max_bins <= 65536, else uint32."""
        _need(sym, torch.uint16, "sym")
        n, F = sym.shape
        rowptr = self.empty((n + 1,), torch.int32)
        ws_bytes = self.lib.gbt_compress_sparse_workspace_bytes(n)
        ws = self.workspace("small", max(ws_bytes, 4096))
        nnz = C.c_int64()
        self._check(self.lib.gbt_compress_sparse_count(self.h, _ptr(sym), n, F, missing_sym, _ptr(rowptr),
                                                       C.byref(nnz), _ptr(ws), ws.numel()))
        cap = int(self.lib.gbt_sparse_capacity(nnz.value))
        width = int(self.lib.gbt_sparse_entry_bytes(F, max_bins))
        if width == 0:
            raise GbtError(EUNSUPPORTED, f"gbt_sparse_entry_bytes rejected F = {F}, max_bins = {max_bins}")
        ent = self.empty((cap,), torch.uint16 if width == 2 else torch.uint32)
        self._check(self.lib.gbt_compress_sparse(self.h, _ptr(sym), n, F, max_bins, missing_sym, _ptr(rowptr),
                                                 nnz.value, _ptr(ent), cap))
        return rowptr, ent, nnz.value

    # -- Sec. 2.5 ------------------------------------------------------------
    def gradients(self, objective: str, margin, label, out=None):
        _need(margin, torch.float32, "margin"); _need(label, torch.float32, "label")
        n = margin.numel()
        gp = out if out is not None else self.empty((n, 2), torch.float32)
        self._check(self.lib.gbt_gradients(self.h, OBJECTIVES[objective], _ptr(margin), _ptr(label), n, _ptr(gp)))
        return gp

    # -- histograms ----------------------------------------------------------
    def gpair_fixed(self, gpair):
        _need(gpair, torch.float32, "gpair")
        n = gpair.shape[0]
        gq = self.empty((n, 2), torch.int32)
        scale = (C.c_double * 2)()
        ws = self.workspace("small", 4096)
        self._check(self.lib.gbt_gpair_fixed(self.h, _ptr(gpair), n, _ptr(gq), scale, _ptr(ws), ws.numel()))
        return gq, (scale[0], scale[1])

    def _rows_ptr(self, row_idx):
        # NULL means "all rows"; an empty list still needs a non-null address
        if row_idx is not None and row_idx.numel() == 0:
            return _ptr(self.workspace("small", 4096))
        return _ptr(row_idx)

    def sum_gpair(self, gq, row_idx=None):
        n_rows = gq.shape[0] if row_idx is None else row_idx.numel()
        out = (C.c_int64 * 2)()
        ws = self.workspace("small", 4096)
        self._check(self.lib.gbt_sum_gpair(self.h, _ptr(gq), self._rows_ptr(row_idx), n_rows, out, _ptr(ws),
                                           ws.numel()))
        return int(out[0]), int(out[1])

    def build_hist(self, packed, bits, n, F, B, missing_sym, gq, row_idx=None, out=None):
        hist = out if out is not None else self.empty((F, B, 2), torch.int64)
        n_rows = 0 if row_idx is None else row_idx.numel()
        self._check(self.lib.gbt_build_hist(self.h, _ptr(packed), bits, n, F, B, missing_sym,
                                            self._rows_ptr(row_idx), n_rows, _ptr(gq), _ptr(hist)))
        return hist

    def build_hist_sparse(self, rowptr, ent, n, F, B, gq, row_begin=0, n_rows=None, out=None):
        hist = out if out is not None else self.empty((F, B, 2), torch.int64)
        self._check(self.lib.gbt_build_hist_sparse(self.h, _ptr(rowptr), _ptr(ent), n, F, B, row_begin,
                                                   n if n_rows is None else n_rows, _ptr(gq), _ptr(hist)))
        return hist

    def hist_subtract(self, parent, child):
        out = torch.empty_like(parent)
        self._check(self.lib.gbt_hist_subtract(self.h, _ptr(parent), _ptr(child), _ptr(out), parent.numel()))
        return out

    def hist_export_f64(self, hist, scale):
        F, B, _ = hist.shape
        out = self.empty((F, B, 2), torch.float64)
        sc = (C.c_double * 2)(*scale)
        self._check(self.lib.gbt_hist_export_f64(self.h, _ptr(hist), F, B, sc, _ptr(out)))
        return out

    # -- split ---------------------------------------------------------------
    def eval_split(self, hist, nb, Gq, Hq, scale, params: Params) -> dict:
        F, B, _ = hist.shape
        sc = (C.c_double * 2)(*scale)
        sp = Split()
        ws = self.workspace("small", 4096)
        self._check(self.lib.gbt_eval_split(self.h, _ptr(hist), _ptr(nb), F, B, Gq, Hq, sc, C.byref(params),
                                            C.byref(sp), _ptr(ws), ws.numel()))
        return {k: getattr(sp, k) for k, _ in Split._fields_}

    # -- partition -----------------------------------------------------------
    def partition(self, packed, bits, n, F, row_idx, begin, end, feature, bin_, default_left, missing_sym) -> int:
        _need(row_idx, torch.int32, "row_idx")
        ws_bytes = self.lib.gbt_partition_workspace_bytes(end - begin)
        ws = self.workspace("partition", ws_bytes)
        nl = C.c_int64()
        self._check(self.lib.gbt_partition(self.h, _ptr(packed), bits, n, F, _ptr(row_idx), begin, end, feature,
                                           bin_, default_left, missing_sym, _ptr(ws), ws.numel(), C.byref(nl)))
        return nl.value

    def partition_static(self, packed, bits, n, F, row_idx, begin, end, feature, bin_, default_left, missing_sym) -> int:
        """gbt_partition_static: the same partition over the library's static scratch array (no workspace)."""
        _need(row_idx, torch.int32, "row_idx")
        nl = C.c_int64()
        self._check(self.lib.gbt_partition_static(self.h, _ptr(packed), bits, n, F, _ptr(row_idx), begin, end, feature,
                                                  bin_, default_left, missing_sym, C.byref(nl)))
        return nl.value

    # -- Alg. 1 --------------------------------------------------------------
    def grow_tree(self, packed, bits, n, F, missing_sym, nb, cuts, gpair, params: Params, want_leaf=True,
                  row_idx_out=None, leaf_out=None, want_rows=True):
        """Returns (tree dict of numpy arrays, row_idx int32 tensor [n], leaf_of_row int32 tensor [n]).
        want_rows=False: the final row order is not produced (row_idx is None), which lets the library
        take its faster partition paths; leaf_of_row is still available (want_leaf)."""
        t = new_tree(params.max_depth)
        ts = _tree_struct(t)
        if not want_rows:
            row_idx = None
        else:
            row_idx = row_idx_out if row_idx_out is not None else self.empty((n,), torch.int32)
        leaf = (leaf_out if leaf_out is not None else self.empty((n,), torch.int32)) if want_leaf else None
        ws_bytes = self.lib.gbt_grow_tree_workspace_bytes(n, F, bits, params.max_bins, params.max_depth)
        if ws_bytes == 0:
            raise GbtError(EINVAL, "gbt_grow_tree_workspace_bytes rejected the shape")
        ws = self.workspace("grow", ws_bytes)
        self._check(self.lib.gbt_grow_tree(self.h, _ptr(packed), bits, n, F, missing_sym, _ptr(nb), _ptr(cuts),
                                           _ptr(gpair), C.byref(params), C.byref(ts), _ptr(row_idx), _ptr(leaf),
                                           _ptr(ws), ws.numel()))
        t["n_nodes"] = int(ts.n_nodes)
        return t, row_idx, leaf

    def boost_round(self, packed, bits, n, F, missing_sym, nb, cuts, label, margin_in, margin_out, gpair, params: Params):
        """Gradients of margin_in, one depth-wise tree, margin_out = margin_in + eta * leaf weight.  Returns the tree."""
        for t_, nm in ((label, "label"), (margin_in, "margin_in"), (margin_out, "margin_out"), (gpair, "gpair")):
            _need(t_, torch.float32, nm)
        t = new_tree(params.max_depth)
        ts = _tree_struct(t)
        ws_bytes = self.lib.gbt_grow_tree_workspace_bytes(n, F, bits, params.max_bins, params.max_depth)
        if ws_bytes == 0:
            raise GbtError(EINVAL, "gbt_grow_tree_workspace_bytes rejected the shape")
        ws = self.workspace("grow", ws_bytes)
        self._check(self.lib.gbt_boost_round(self.h, _ptr(packed), bits, n, F, missing_sym, _ptr(nb), _ptr(cuts),
                                             _ptr(label), _ptr(margin_in), _ptr(margin_out), _ptr(gpair),
                                             C.byref(params), C.byref(ts), _ptr(ws), ws.numel()))
        t["n_nodes"] = int(ts.n_nodes)
        return t

    def grow_tree_sparse(self, rowptr, ent, n, nnz, F, nb, cuts, gpair, params: Params, want_leaf=True,
                         want_rows=True):
        """grow_tree over sparse rows (compress_sparse); returns what grow_tree returns."""
        t = new_tree(params.max_depth)
        ts = _tree_struct(t)
        row_idx = self.empty((n,), torch.int32) if want_rows else None
        leaf = self.empty((n,), torch.int32) if want_leaf else None
        ws_bytes = self.lib.gbt_grow_tree_sparse_workspace_bytes(n, nnz, F, params.max_bins, params.max_depth)
        if ws_bytes == 0:
            raise GbtError(EINVAL, "gbt_grow_tree_sparse_workspace_bytes rejected the shape")
        ws = self.workspace("grow", ws_bytes)
        self._check(self.lib.gbt_grow_tree_sparse(self.h, _ptr(rowptr), _ptr(ent), n, nnz, F, _ptr(nb), _ptr(cuts),
                                                  _ptr(gpair), C.byref(params), C.byref(ts), _ptr(row_idx),
                                                  _ptr(leaf), _ptr(ws), ws.numel()))
        t["n_nodes"] = int(ts.n_nodes)
        return t, row_idx, leaf

    def grow_tree_sparse_lossguide(self, rowptr, ent, n, nnz, F, nb, cuts, gpair, params: Params, max_leaves,
                                   want_leaf=True, want_rows=True):
        """Loss-guided growth (Sec. 2.3) over sparse rows; returns what grow_tree returns."""
        t = new_tree_leaves(max_leaves)
        ts = _tree_struct(t)
        row_idx = self.empty((n,), torch.int32) if want_rows else None
        leaf = self.empty((n,), torch.int32) if want_leaf else None
        ws_bytes = self.lib.gbt_grow_tree_sparse_lossguide_workspace_bytes(n, nnz, F, params.max_bins, max_leaves)
        if ws_bytes == 0:
            raise GbtError(EINVAL, "gbt_grow_tree_sparse_lossguide_workspace_bytes rejected the shape")
        ws = self.workspace("grow", ws_bytes)
        self._check(self.lib.gbt_grow_tree_sparse_lossguide(self.h, _ptr(rowptr), _ptr(ent), n, nnz, F, _ptr(nb),
                                                            _ptr(cuts), _ptr(gpair), C.byref(params), max_leaves,
                                                            C.byref(ts), _ptr(row_idx), _ptr(leaf), _ptr(ws), ws.numel()))
        t["n_nodes"] = int(ts.n_nodes)
        return t, row_idx, leaf

    def grow_tree_lossguide(self, packed, bits, n, F, missing_sym, nb, cuts, gpair, params: Params, max_leaves,
                            want_leaf=True, want_rows=True):
        """Loss-guided growth (Sec. 2.3); returns what grow_tree returns."""
        t = new_tree_leaves(max_leaves)
        ts = _tree_struct(t)
        row_idx = self.empty((n,), torch.int32) if want_rows else None
        leaf = self.empty((n,), torch.int32) if want_leaf else None
        ws_bytes = self.lib.gbt_grow_tree_lossguide_workspace_bytes(n, F, bits, params.max_bins, max_leaves)
        if ws_bytes == 0:
            raise GbtError(EINVAL, "gbt_grow_tree_lossguide_workspace_bytes rejected the shape")
        ws = self.workspace("grow", ws_bytes)
        self._check(self.lib.gbt_grow_tree_lossguide(self.h, _ptr(packed), bits, n, F, missing_sym, _ptr(nb),
                                                     _ptr(cuts), _ptr(gpair), C.byref(params), max_leaves,
                                                     C.byref(ts), _ptr(row_idx), _ptr(leaf), _ptr(ws), ws.numel()))
        t["n_nodes"] = int(ts.n_nodes)
        return t, row_idx, leaf

    def grow_tree_path(self, F, bits, max_bins, track_rows=True):
        """0: three-launch partition, 1: one-launch partition, 2: partition + histogram in one launch."""
        r = self.lib.gbt_grow_tree_path(self.h, F, bits, max_bins, 1 if track_rows else 0)
        if r < 0:
            self._check(r)
        return r

    # -- Sec. 2.4 ------------------------------------------------------------
    def predict_sparse(self, trees, margin, eta: float, rowptr, ent, n, F, max_bins):
        arr = (Tree * len(trees))(*[_tree_struct(t) for t in trees])
        ws_bytes = self.lib.gbt_predict_workspace_bytes(arr, len(trees))
        ws = self.workspace("predict", ws_bytes)
        self._check(self.lib.gbt_predict_sparse(self.h, arr, len(trees), _ptr(rowptr), _ptr(ent), n, F, max_bins, eta,
                                                _ptr(margin), _ptr(ws), ws.numel()))
        return margin

    def predict(self, trees, margin, eta: float, *, packed=None, bits=0, missing_sym=0, X=None, n=None, F=None):
        arr = (Tree * len(trees))(*[_tree_struct(t) for t in trees])
        if X is not None:
            n, F = X.shape
        ws_bytes = self.lib.gbt_predict_workspace_bytes(arr, len(trees))
        ws = self.workspace("predict", ws_bytes)
        self._check(self.lib.gbt_predict(self.h, arr, len(trees), _ptr(packed), bits, missing_sym, _ptr(X), n, F,
                                         eta, _ptr(margin), _ptr(ws), ws.numel()))
        return margin
