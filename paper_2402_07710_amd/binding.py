"""ctypes binding of libsc.so: the same calls as include/sc.h, taking torch tensors.

Argument marshalling only - every step of the path runs in the library's HIP kernels.  PyTorch
supplies device memory (tensors) and the stream.  There is no CPU fallback: if the library has
not been built, or no GPU is present when a call needs one, the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SC_LIB_PATH", os.path.join(HERE, "libsc.so"))   # override: development builds

SC_OK, SC_EINVAL, SC_ERANGE, SC_EDUP, SC_ECAP, SC_EHIP, SC_EFULL = 0, -1, -2, -3, -4, -5, -6
SC_SUBM, SC_STRIDED, SC_INVERSE = 0, 1, 2
SC_F32, SC_F16, SC_BF16 = 0, 1, 2
SC_COORD_MAX, SC_N_MAX, SC_K_MAX = 65534, 1 << 26, 7
SC_BATCH_MAX, SC_HASH_EPOCH_MAX = 255, 254
MODES = {"subm": SC_SUBM, "strided": SC_STRIDED, "inverse": SC_INVERSE,
         SC_SUBM: SC_SUBM, SC_STRIDED: SC_STRIDED, SC_INVERSE: SC_INVERSE}
DTYPES = {"f32": SC_F32, "f16": SC_F16, "bf16": SC_BF16,
          torch.float32: SC_F32, torch.float16: SC_F16, torch.bfloat16: SC_BF16}
TORCH_DTYPES = {SC_F32: torch.float32, SC_F16: torch.float16, SC_BF16: torch.bfloat16}

# every symbol include/sc.h declares
SYMBOLS = ["sc_hash_bytes", "sc_hash_build", "sc_hash_rebuild", "sc_hash_lookup", "sc_out_bound", "sc_kmap_bytes",
           "sc_kmap_scratch_bytes", "sc_kmap_build", "sc_kmap_transpose", "sc_conv_workspace_bytes", "sc_conv_fwd",
           "sc_counts_read", "sc_kmap_export", "sc_strerror", "sc_profile_enable", "sc_profile_read",
           "sc_grid_bytes", "sc_grid_clear", "sc_grid_build", "sc_grid_lookup", "sc_kmap_build_grid",
           "sc_conv_fwd_grid", "sc_conv_up_fwd", "sc_kmap_build_noalloc", "sc_profile_mfma_peak",
           "sc_conv_packed_bytes", "sc_conv_weight_pack", "sc_conv_fwd_packed", "sc_hash_probe_slot"]


class ScCounts(ctypes.Structure):
    _fields_ = [("n_in", ctypes.c_int64), ("n_out", ctypes.c_int64), ("n_pairs", ctypes.c_int64),
                ("per_offset", ctypes.c_int32 * 343), ("status", ctypes.c_int32)]


COUNTS_BYTES = ctypes.sizeof(ScCounts)


class ScProfileEntry(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("launches", ctypes.c_int64), ("total_ms", ctypes.c_double),
                ("median_ms", ctypes.c_double)]


class ScError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


_lib = None


def load(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load libsc.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(f"{LIB_PATH} has not been built")
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    sig = {
        "sc_hash_bytes": (sz, [i64]),
        "sc_hash_build": (i32, [vp, i64, vp, sz, vp, vp]),
        "sc_hash_rebuild": (i32, [vp, i64, vp, sz, i32, vp, vp]),
        "sc_conv_up_fwd": (i32, [vp, i64, vp, vp, vp, sz, vp, i32, i32, i32, i32, i32, vp]),
        "sc_hash_lookup": (i32, [vp, i64, vp, i64, vp, vp]),
        "sc_out_bound": (i64, [i64, i32, i32, i32]),
        "sc_kmap_bytes": (sz, [i64, i32, i32, i32]),
        "sc_kmap_scratch_bytes": (sz, [i64, i32, i32, i32]),
        "sc_kmap_build": (i32, [vp, i64, vp, i32, i32, i32, vp, vp, sz, vp, sz, vp, vp]),
        "sc_kmap_build_noalloc": (i32, [vp, i64, vp, i32, i32, i32, vp, vp, sz, vp, vp]),
        "sc_kmap_transpose": (i32, [vp, i64, i32, i32, vp, vp, sz, vp]),
        "sc_conv_workspace_bytes": (sz, [i32, i32, i32, i32]),
        "sc_conv_fwd": (i32, [vp, i64, vp, vp, i64, vp, sz, vp, i32, i32, i32, i32, i32, i32, i32, vp, sz, vp]),
        "sc_conv_packed_bytes": (sz, [i32, i32, i32, i32]),
        "sc_conv_weight_pack": (i32, [vp, i32, i32, i32, i32, vp, sz, vp]),
        "sc_conv_fwd_packed": (i32, [vp, i64, vp, vp, i64, vp, sz, vp, i32, i32, i32, i32, i32, i32, i32, vp]),
        "sc_counts_read": (i32, [vp, ctypes.POINTER(ScCounts), vp, i64, i32, i32, i32, vp]),
        "sc_kmap_export": (i32, [vp, i64, i32, i32, i32, ctypes.POINTER(ScCounts), vp, vp, vp, vp]),
        "sc_strerror": (ctypes.c_char_p, [i32]),
        "sc_hash_probe_slot": (i64, [i32, i32, i32, i32, ctypes.c_uint32, i64]),
        "sc_profile_enable": (i32, [i32]),
        "sc_profile_read": (i32, [ctypes.POINTER(ScProfileEntry), i32]),
        "sc_profile_mfma_peak": (i32, [ctypes.POINTER(ctypes.c_double)]),
        "sc_grid_bytes": (sz, [i32, i32, i32, i32]),
        "sc_grid_clear": (i32, [vp, sz, i32, i32, i32, i32, vp]),
        "sc_grid_build": (i32, [vp, i64, vp, sz, i32, i32, i32, i32, ctypes.c_uint32, vp, vp]),
        "sc_grid_lookup": (i32, [vp, i32, i32, i32, i32, ctypes.c_uint32, vp, i64, vp, vp]),
        "sc_kmap_build_grid": (i32, [vp, i64, vp, sz, i32, i32, i32, i32, ctypes.c_uint32, i32, vp, sz, vp, vp]),
        "sc_conv_fwd_grid": (i32, [vp, vp, i64, vp, sz, i32, i32, i32, i32, ctypes.c_uint32, vp, vp, i32, i32, i32, i32, i32,
                                   vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().sc_strerror(code).decode()


def _check(code: int, what: str):
    if code != SC_OK:
        raise ScError(code, what)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


# ---- the calls of sc.h, same names ----------------------------------------------------------
def sc_hash_bytes(n: int) -> int:
    return load().sc_hash_bytes(n)


def sc_out_bound(n: int, K: int, stride: int, mode) -> int:
    return load().sc_out_bound(n, K, stride, MODES[mode])


def sc_kmap_bytes(n: int, K: int, stride: int, mode) -> int:
    return load().sc_kmap_bytes(n, K, stride, MODES[mode])


def sc_kmap_scratch_bytes(n: int, K: int, stride: int, mode) -> int:
    return load().sc_kmap_scratch_bytes(n, K, stride, MODES[mode])


def sc_conv_workspace_bytes(K: int, C_in: int, C_out: int, dtype) -> int:
    return load().sc_conv_workspace_bytes(K, C_in, C_out, DTYPES[dtype])


def sc_hash_build(coords, table, counts, stream=None):
    """coords int32 [n,4] (device), table uint8 [>= sc_hash_bytes(n)], counts uint8 [COUNTS_BYTES]."""
    n = coords.shape[0]
    _check(load().sc_hash_build(_ptr(coords), n, _ptr(table), table.numel() * table.element_size(),
                                _ptr(counts), _stream(stream)), "sc_hash_build")


def sc_hash_rebuild(coords, table, epoch, counts, stream=None):
    """Build again, without the filling pass, into a table that sc_hash_build initialised (same n)."""
    n = coords.shape[0]
    _check(load().sc_hash_rebuild(_ptr(coords), n, _ptr(table), table.numel() * table.element_size(), epoch,
                                  _ptr(counts), _stream(stream)), "sc_hash_rebuild")


def sc_hash_lookup(table, n_table, query, rows, stream=None):
    _check(load().sc_hash_lookup(_ptr(table), n_table, _ptr(query), query.shape[0], _ptr(rows),
                                 _stream(stream)), "sc_hash_lookup")


def sc_kmap_build(coords, table, K, stride, mode, out_coords, kmap, scratch, counts, stream=None):
    n = coords.shape[0]
    _check(load().sc_kmap_build(_ptr(coords), n, _ptr(table), K, stride, MODES[mode], _ptr(out_coords),
                                _ptr(kmap), kmap.numel() * kmap.element_size(),
                                _ptr(scratch), 0 if scratch is None else scratch.numel() * scratch.element_size(),
                                _ptr(counts), _stream(stream)), "sc_kmap_build")


def sc_kmap_build_noalloc(coords, table, K, stride, mode, out_coords, kmap, counts, stream=None):
    """sc_kmap_build with the scratch buffer inside the library (no device allocation anywhere)."""
    n = coords.shape[0]
    _check(load().sc_kmap_build_noalloc(_ptr(coords), n, _ptr(table), K, stride, MODES[mode], _ptr(out_coords),
                                        _ptr(kmap), kmap.numel() * kmap.element_size(), _ptr(counts),
                                        _stream(stream)), "sc_kmap_build_noalloc")


def sc_grid_bytes(B: int, X: int, Y: int, Z: int) -> int:
    return load().sc_grid_bytes(B, X, Y, Z)


def sc_grid_clear(grid, dims, stream=None):
    _check(load().sc_grid_clear(_ptr(grid), grid.numel() * grid.element_size(), *dims, _stream(stream)), "sc_grid_clear")


def sc_grid_build(coords, grid, dims, epoch, counts, stream=None):
    """coords int32 [n,4] (device), grid uint8 [>= sc_grid_bytes(*dims)], dims = (B, X, Y, Z)."""
    _check(load().sc_grid_build(_ptr(coords), coords.shape[0], _ptr(grid), grid.numel() * grid.element_size(), *dims,
                                epoch, _ptr(counts), _stream(stream)), "sc_grid_build")


def sc_grid_lookup(grid, dims, epoch, query, rows, stream=None):
    _check(load().sc_grid_lookup(_ptr(grid), *dims, epoch, _ptr(query), query.shape[0], _ptr(rows), _stream(stream)),
           "sc_grid_lookup")


def sc_kmap_build_grid(coords, grid, dims, epoch, K, kmap, counts, stream=None):
    _check(load().sc_kmap_build_grid(_ptr(coords), coords.shape[0], _ptr(grid), grid.numel() * grid.element_size(),
                                     *dims, epoch, K, _ptr(kmap), kmap.numel() * kmap.element_size(), _ptr(counts),
                                     _stream(stream)), "sc_kmap_build_grid")


def sc_conv_up_fwd(feat_coarse, n_map, weight, feat_fine, kmap, counts, K, stream=None):
    """Inverse layer of a K == stride layer from that layer's own map: feat_coarse [n_out, C_in],
    weight [K^3, C_in, C_out], feat_fine [n_map, C_out]."""
    C_in, C_out = weight.shape[1], weight.shape[2]
    if tuple(weight.shape) != (K ** 3, C_in, C_out) or weight.dtype != feat_coarse.dtype or \
            feat_coarse.shape[1] != C_in or tuple(feat_fine.shape) != (n_map, C_out):
        raise ScError(SC_EINVAL, "sc_conv_up_fwd")
    _check(load().sc_conv_up_fwd(_ptr(feat_coarse), n_map, _ptr(weight), _ptr(feat_fine), _ptr(kmap),
                                 kmap.numel() * kmap.element_size(), _ptr(counts), K, C_in, C_out,
                                 DTYPES[feat_coarse.dtype], DTYPES[feat_fine.dtype], _stream(stream)), "sc_conv_up_fwd")


def sc_conv_fwd_grid(feat_in, coords, grid, dims, epoch, weight, feat_out, K, workspace, stream=None):
    """Fused 3x3x3 submanifold layer over the dense table: no kernel map."""
    C_in, C_out = weight.shape[1], weight.shape[2]
    _check(load().sc_conv_fwd_grid(_ptr(feat_in), _ptr(coords), coords.shape[0], _ptr(grid),
                                   grid.numel() * grid.element_size(), *dims, epoch, _ptr(weight), _ptr(feat_out), K,
                                   C_in, C_out, DTYPES[feat_in.dtype], DTYPES[feat_out.dtype], _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)), "sc_conv_fwd_grid")


def sc_kmap_transpose(kmap, n, K, stride, counts, kmap_inv, stream=None):
    _check(load().sc_kmap_transpose(_ptr(kmap), n, K, stride, _ptr(counts), _ptr(kmap_inv),
                                    kmap_inv.numel() * kmap_inv.element_size(), _stream(stream)), "sc_kmap_transpose")


def sc_conv_fwd(feat_in, weight, feat_out, kmap, counts, K, stride, mode, workspace=None, stream=None, n_map=None):
    """feat_in [rows,C_in], weight [K^3,C_in,C_out] (same dtype), feat_out [n_out_cap,C_out];
    n_map = the n the map was built with (default: rows of feat_in)."""
    n_in, C_in = feat_in.shape
    n_out_cap, C_out = feat_out.shape
    if n_map is None:
        n_map = n_in
    if tuple(weight.shape) != (K ** 3, C_in, C_out) or weight.dtype != feat_in.dtype:
        raise ValueError("weight must be [K^3, C_in, C_out] in the feature dtype")
    _check(load().sc_conv_fwd(_ptr(feat_in), n_map, _ptr(weight), _ptr(feat_out), n_out_cap, _ptr(kmap),
                              kmap.numel() * kmap.element_size(), _ptr(counts), K, stride, MODES[mode],
                              C_in, C_out, DTYPES[feat_in.dtype], DTYPES[feat_out.dtype], _ptr(workspace),
                              0 if workspace is None else workspace.numel() * workspace.element_size(),
                              _stream(stream)), "sc_conv_fwd")


def sc_conv_packed_bytes(K: int, C_in: int, C_out: int, dtype) -> int:
    return load().sc_conv_packed_bytes(K, C_in, C_out, DTYPES[dtype])


def sc_conv_weight_pack(weight, K, packed=None, stream=None):
    """weight [K^3, C_in, C_out] -> the packed form sc_conv_fwd_packed takes (a uint8 tensor; allocated
    here unless `packed` is given)."""
    C_in, C_out = weight.shape[1], weight.shape[2]
    if tuple(weight.shape) != (K ** 3, C_in, C_out):
        raise ValueError("weight must be [K^3, C_in, C_out]")
    if packed is None:
        packed = torch.empty(max(sc_conv_packed_bytes(K, C_in, C_out, weight.dtype), 16), dtype=torch.uint8,
                             device=weight.device)
    _check(load().sc_conv_weight_pack(_ptr(weight), K, C_in, C_out, DTYPES[weight.dtype], _ptr(packed),
                                      packed.numel() * packed.element_size(), _stream(stream)), "sc_conv_weight_pack")
    return packed


def sc_conv_fwd_packed(feat_in, packed, C_out, feat_out, kmap, counts, K, stride, mode, stream=None, n_map=None):
    """sc_conv_fwd with weights packed by sc_conv_weight_pack."""
    n_in, C_in = feat_in.shape
    n_out_cap = feat_out.shape[0]
    if n_map is None:
        n_map = n_in
    if feat_out.shape[1] != C_out:
        raise ValueError("feat_out must have C_out columns")
    _check(load().sc_conv_fwd_packed(_ptr(feat_in), n_map, _ptr(packed), _ptr(feat_out), n_out_cap, _ptr(kmap),
                                     kmap.numel() * kmap.element_size(), _ptr(counts), K, stride, MODES[mode],
                                     C_in, C_out, DTYPES[feat_in.dtype], DTYPES[feat_out.dtype], _stream(stream)),
           "sc_conv_fwd_packed")


def sc_counts_read(counts, kmap=None, n=0, K=1, stride=1, mode="subm", stream=None, check=True) -> ScCounts:
    h = ScCounts()
    rc = load().sc_counts_read(_ptr(counts), ctypes.byref(h), _ptr(kmap), n, K, stride, MODES[mode], _stream(stream))
    if check:
        _check(rc, "sc_counts_read")
    return h


def sc_kmap_export(kmap, n, K, stride, mode, h_counts: ScCounts, stream=None):
    """Plain rulebook of a map: (pairs_in [P], pairs_out [P], offset_start [K^3+1]) int32 device tensors."""
    dev = kmap.device
    P = int(h_counts.n_pairs)
    pin = torch.empty(max(P, 1), dtype=torch.int32, device=dev)
    pout = torch.empty(max(P, 1), dtype=torch.int32, device=dev)
    ost = torch.empty(K ** 3 + 1, dtype=torch.int32, device=dev)
    _check(load().sc_kmap_export(_ptr(kmap), n, K, stride, MODES[mode], ctypes.byref(h_counts), _ptr(pin), _ptr(pout),
                                 _ptr(ost), _stream(stream)), "sc_kmap_export")
    return pin[:P], pout[:P], ost


def sc_profile_enable(enable: bool):
    _check(load().sc_profile_enable(1 if enable else 0), "sc_profile_enable")


def sc_profile_read() -> dict:
    """{kernel name: (launches, total ms, median ms)} for the kernels that ran since sc_profile_enable(True)."""
    arr = (ScProfileEntry * 32)()
    n = load().sc_profile_read(arr, 32)
    if n < 0:
        raise ScError(n, "sc_profile_read")
    return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].total_ms), float(arr[i].median_ms))
            for i in range(n)}


def sc_profile_mfma_peak() -> float:
    """Sustained TFLOP/s of a register-operand fp16 MFMA loop on the current device."""
    v = ctypes.c_double(0.0)
    _check(load().sc_profile_mfma_peak(ctypes.byref(v)), "sc_profile_mfma_peak")
    return v.value


# ---- buffers for one layer -------------------------------------------------------------------
class LayerBuffers:
    """All device buffers one layer needs, allocated once (torch tensors), plus the three calls
    in order.  Holds no arithmetic: it sizes buffers with the library's own *_bytes calls."""

    def __init__(self, n: int, K: int, stride: int, mode, C_in: int, C_out: int, dtype, out_dtype=None,
                 device="cuda:0", grid_dims=None):
        """grid_dims = (B, X, Y, Z): use the dense location table over that box instead of the hash
        table (submanifold layers only)."""
        self.n, self.K, self.stride, self.mode = n, K, stride, MODES[mode]
        self.C_in, self.C_out = C_in, C_out
        self.dtype = TORCH_DTYPES[DTYPES[dtype]]
        self.out_dtype = self.dtype if out_dtype is None else TORCH_DTYPES[DTYPES[out_dtype]]
        self.bound = sc_out_bound(n, K, stride, mode)
        if self.bound < 0:
            raise ScError(SC_EINVAL, "sc_out_bound")
        u8 = dict(dtype=torch.uint8, device=device)
        self.grid_dims, self.epoch = grid_dims, 0
        self._hash_n = None          # rows of the sc_hash_build that initialised the hash table
        if grid_dims is None:
            self.table = torch.empty(max(sc_hash_bytes(n), 16), **u8)
        else:
            if self.mode != SC_SUBM or sc_grid_bytes(*grid_dims) == 0:
                raise ScError(SC_EINVAL, "sc_grid_bytes")
            self.table = torch.empty(sc_grid_bytes(*grid_dims), **u8)
            sc_grid_clear(self.table, grid_dims)
        self.kmap = torch.empty(max(sc_kmap_bytes(n, K, stride, mode), 16), **u8)
        self.scratch = torch.empty(max(sc_kmap_scratch_bytes(n, K, stride, mode), 16), **u8)
        self.workspace = torch.empty(max(sc_conv_workspace_bytes(K, C_in, C_out, dtype), 16), **u8)
        self.counts = torch.zeros(COUNTS_BYTES + 8, **u8)
        # submanifold outputs are the inputs themselves: no copy is asked for
        self.out_coords = (None if self.mode == SC_SUBM else
                           torch.empty((max(self.bound, 1), 4), dtype=torch.int32, device=device))
        self.feat_out = torch.empty((max(self.bound, 1), C_out), dtype=self.out_dtype, device=device)

    def hash_build(self, coords, stream=None):
        """Location table over `coords`: the hash table, or the dense array if grid_dims was given."""
        if self.grid_dims is None:
            # the first build fills the table; later ones of the same size only move to a new epoch
            if self._hash_n == coords.shape[0] and self.epoch < SC_HASH_EPOCH_MAX:
                self.epoch += 1
                sc_hash_rebuild(coords, self.table, self.epoch, self.counts, stream)
            else:
                self._hash_n, self.epoch = coords.shape[0], 0
                sc_hash_build(coords, self.table, self.counts, stream)
        else:
            self.epoch += 1
            if self.epoch >= 1 << 32:
                sc_grid_clear(self.table, self.grid_dims, stream)
                self.epoch = 1
            sc_grid_build(coords, self.table, self.grid_dims, self.epoch, self.counts, stream)

    def forget_table(self):
        """Make the next hash_build a full sc_hash_build (fill + inserts), as on a fresh table."""
        self._hash_n = None

    def kmap_build(self, coords, stream=None, standalone=False):
        """standalone (strided layers): no location table is passed, the build starts the counts
        block itself and repeated input coordinates go unnoticed."""
        if self.grid_dims is not None:
            sc_kmap_build_grid(coords, self.table, self.grid_dims, self.epoch, self.K, self.kmap, self.counts, stream)
            self.out_coords = coords
            return
        sc_kmap_build(coords, None if standalone else self.table, self.K, self.stride, self.mode,
                      None if self.mode == SC_SUBM else self.out_coords, self.kmap,
                      self.scratch, self.counts, stream)
        if self.mode == SC_SUBM:
            self.out_coords = coords

    def conv_fwd(self, feat_in, weight, stream=None):
        sc_conv_fwd(feat_in, weight, self.feat_out, self.kmap, self.counts, self.K, self.stride, self.mode,
                    self.workspace, stream)

    def conv_fwd_packed(self, feat_in, packed, stream=None):
        """The convolution with weights packed once by sc_conv_weight_pack."""
        sc_conv_fwd_packed(feat_in, packed, self.C_out, self.feat_out, self.kmap, self.counts, self.K, self.stride,
                           self.mode, stream)

    def layer_fused(self, coords, feat_in, weight, stream=None):
        """Dense table + fused look-up and convolution (3x3x3 submanifold layers, grid_dims given)."""
        self.hash_build(coords, stream)
        sc_conv_fwd_grid(feat_in, coords, self.table, self.grid_dims, self.epoch, weight, self.feat_out, self.K,
                         self.workspace, stream)
        self.out_coords = coords

    def layer(self, coords, feat_in, weight, stream=None):
        self.hash_build(coords, stream)
        self.kmap_build(coords, stream)
        self.conv_fwd(feat_in, weight, stream)

    def read_counts(self, with_pairs=True, stream=None, check=True) -> ScCounts:
        return sc_counts_read(self.counts, self.kmap if with_pairs else None, self.n, self.K, self.stride,
                              self.mode, stream, check)

    def export(self, h_counts=None, stream=None):
        if h_counts is None:
            h_counts = self.read_counts(stream=stream)
        return sc_kmap_export(self.kmap, self.n, self.K, self.stride, self.mode, h_counts, stream)
