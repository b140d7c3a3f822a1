"""CPU oracle for the sparse-convolution path — TEST INFRASTRUCTURE ONLY.

Thin ctypes front for `sc_oracle.cpp` (std::map lookups, one triple loop per offset, fp64).
Only tests, the smoke check and the benchmark's cpu_baseline leg import this package; it
imports nothing from the GPU package and the GPU package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import numpy as np

from . import build as _build

SUBM, STRIDED = 0, 1
_MODES = {"subm": SUBM, "strided": STRIDED, SUBM: SUBM, STRIDED: STRIDED}
_ERRORS = {-1: "invalid argument", -2: "duplicate input coordinate",
           -3: "negative coordinate", -4: "output buffer too small"}

_lib = None


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle: {_ERRORS.get(code, code)}")
        self.code = code


def _ptr(a, t):
    return a.ctypes.data_as(ctypes.POINTER(t))


class Oracle:
    """The oracle library loaded from one shared object (the default build, or another build of
    the same source that a test made)."""

    def __init__(self, lib_path: str | None = None):
        lib = ctypes.CDLL(lib_path or _build.build())
        i32p, i64p, f64p = (ctypes.POINTER(t) for t in (ctypes.c_int32, ctypes.c_int64, ctypes.c_double))
        lib.sc_oracle_kmap.restype = ctypes.c_int
        lib.sc_oracle_kmap.argtypes = [i32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       i32p, ctypes.c_int64, i64p, i32p, i32p, ctypes.c_int64, i64p]
        lib.sc_oracle_conv.restype = ctypes.c_int
        lib.sc_oracle_conv.argtypes = [f64p, ctypes.c_int64, f64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       i32p, i32p, i64p, f64p, ctypes.c_int64, ctypes.c_int]
        self._lib = lib

    def kmap(self, coords, K: int, stride: int, mode) -> dict:
        """Kernel map of one layer.  Returns out_coords [N_out,4] int32, pair_in / pair_out [P]
        int32 grouped by offset, offset_start [K³+1] int64."""
        coords = np.ascontiguousarray(coords, dtype=np.int32).reshape(-1, 4)
        n = len(coords)
        mode = _MODES[mode]
        K3 = K ** 3
        reach = (-(-K // stride)) ** 3 if mode == STRIDED else 1     # outputs one input can touch
        out_cap = max(1, n * reach)
        pair_cap = max(1, n * (K3 if mode == SUBM else reach))
        out_coords = np.empty((out_cap, 4), dtype=np.int32)
        pair_in = np.empty(pair_cap, dtype=np.int32)
        pair_out = np.empty(pair_cap, dtype=np.int32)
        offset_start = np.zeros(K3 + 1, dtype=np.int64)
        n_out = ctypes.c_int64(0)
        rc = self._lib.sc_oracle_kmap(
            _ptr(coords, ctypes.c_int32), n, K, stride, mode,
            _ptr(out_coords, ctypes.c_int32), out_cap, ctypes.byref(n_out),
            _ptr(pair_in, ctypes.c_int32), _ptr(pair_out, ctypes.c_int32), pair_cap,
            _ptr(offset_start, ctypes.c_int64))
        if rc != 0:
            raise OracleError(rc)
        P = int(offset_start[K3])
        return dict(K=K, stride=stride, mode=mode, n_in=n, n_out=n_out.value,
                    out_coords=out_coords[:n_out.value].copy(),
                    pair_in=pair_in[:P].copy(), pair_out=pair_out[:P].copy(), offset_start=offset_start)

    def conv(self, feat_in, weight, km: dict, threads: int = 1) -> np.ndarray:
        """Output features [N_out, C_out] in float64 from a kernel map `km` (as made by kmap)."""
        feat_in = np.ascontiguousarray(feat_in, dtype=np.float64)
        weight = np.ascontiguousarray(weight, dtype=np.float64)
        n_in, C_in = feat_in.shape
        K3, wc_in, C_out = weight.shape
        if wc_in != C_in or K3 != km["K"] ** 3 or n_in != km["n_in"]:
            raise ValueError("shape mismatch between features, weights and kernel map")
        out = np.empty((km["n_out"], C_out), dtype=np.float64)
        pin = np.ascontiguousarray(km["pair_in"], dtype=np.int32)
        pout = np.ascontiguousarray(km["pair_out"], dtype=np.int32)
        ost = np.ascontiguousarray(km["offset_start"], dtype=np.int64)
        rc = self._lib.sc_oracle_conv(
            _ptr(feat_in, ctypes.c_double), n_in, _ptr(weight, ctypes.c_double), K3, C_in, C_out,
            _ptr(pin, ctypes.c_int32), _ptr(pout, ctypes.c_int32), _ptr(ost, ctypes.c_int64),
            _ptr(out, ctypes.c_double), km["n_out"], threads)
        if rc != 0:
            raise OracleError(rc)
        return out

    def sparse_conv(self, coords, feat_in, weight, K: int, stride: int, mode, threads: int = 1):
        """Whole layer: (out_coords, feat_out float64, kernel map)."""
        km = self.kmap(coords, K, stride, mode)
        return km["out_coords"], self.conv(feat_in, weight, km, threads), km


_default = None


def default() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle()
    return _default


def kmap(coords, K, stride, mode):
    return default().kmap(coords, K, stride, mode)


def conv(feat_in, weight, km, threads=1):
    return default().conv(feat_in, weight, km, threads)


def sparse_conv(coords, feat_in, weight, K, stride, mode, threads=1):
    return default().sparse_conv(coords, feat_in, weight, K, stride, mode, threads)


def transpose_map(km: dict) -> dict:
    """Kernel map of the inverse (up-sampling) layer of Section III-E: the same pairs with input
    and output swapped (a fine row receives from its coarse parent through W[k], k = the fine
    row's place in the kernel).  Inside one offset the pairs are ordered by the new output row."""
    ost = np.asarray(km["offset_start"])
    pin = np.empty_like(km["pair_in"])
    pout = np.empty_like(km["pair_out"])
    for k in range(len(ost) - 1):
        sl = slice(ost[k], ost[k + 1])
        order = np.argsort(km["pair_in"][sl], kind="stable")
        pin[sl] = km["pair_out"][sl][order]
        pout[sl] = km["pair_in"][sl][order]
    return dict(K=km["K"], stride=km["stride"], mode=km["mode"], n_in=km["n_out"], n_out=km["n_in"],
                out_coords=None, pair_in=pin, pair_out=pout, offset_start=ost.copy())


def canonical_pairs(km: dict):
    """Order-independent form of a kernel map: output sites sorted by (b,x,y,z) and renumbered,
    then every offset's pairs sorted by (out, in).  Returns (sorted out_coords, list of [P_k,2]
    int64 arrays (in, out) per offset)."""
    oc = np.asarray(km["out_coords"]).reshape(-1, 4)
    order = np.lexsort((oc[:, 3], oc[:, 2], oc[:, 1], oc[:, 0]))
    rank = np.empty(len(oc), dtype=np.int64)
    rank[order] = np.arange(len(oc))
    ost = np.asarray(km["offset_start"])
    per_k = []
    for k in range(len(ost) - 1):
        i = np.asarray(km["pair_in"][ost[k]:ost[k + 1]], dtype=np.int64)
        o = rank[np.asarray(km["pair_out"][ost[k]:ost[k + 1]], dtype=np.int64)]
        s = np.lexsort((i, o))
        per_k.append(np.stack([i[s], o[s]], axis=1))
    return oc[order], per_k
