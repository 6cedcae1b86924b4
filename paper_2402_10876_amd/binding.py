"""ctypes binding with the same names as the C ABI.  Argument marshalling only:
every step of the path runs inside libtwgemm.so.  The library is loaded from
the package directory and is never built here; a missing library is an error
(there is no fallback path)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

PATTERN_TW, PATTERN_TVW, PATTERN_TEW = 0, 1, 2
LAYOUT_KM, LAYOUT_MK = 0, 1
DTYPE_F16, DTYPE_I8 = 0, 1

EXPORTED_SYMBOLS = [
    "tw_pack_host", "tw_upload", "tw_pack", "tw_pack_dev", "tw_prune_dev",
    "tw_prune_workspace_bytes", "tw_prune_dev_static", "tw_concat", "tw_gemm", "tw_dense_gemm", "tw_export",
    "tw_unpack", "tw_free", "tw_status_str", "tw_set_option", "tw_flop_counts",
    "tw_pack_i8_host", "tw_pack_i8", "tw_gemm_i8", "tw_dense_gemm_i8", "tw_conv_bind", "tw_conv_free", "tw_conv_gemm", "tw_conv_gemm_i8", "tw_calibrate",
    "tw_gemm_ex", "tw_launch_opts_init", "tw_gemm_workspace_bytes", "tw_workspace_init",
]

_lib = None


class TwError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {lib().tw_status_str(status).decode()} (status {status})")


class _View(C.Structure):
    _fields_ = [("K", C.c_int32), ("N", C.c_int32), ("G", C.c_int32), ("pattern", C.c_int32),
                ("n_kept", C.c_int32), ("n_tiles", C.c_int32),
                ("col_idx", C.POINTER(C.c_int32)), ("cto_n", C.POINTER(C.c_int32)),
                ("tile_k_off", C.POINTER(C.c_int32)), ("row_idx", C.POINTER(C.c_int32)),
                ("cto_k", C.POINTER(C.c_int32)), ("val_off", C.POINTER(C.c_int64)),
                ("values", C.POINTER(C.c_uint16)), ("meta_off", C.POINTER(C.c_int64)),
                ("meta", C.POINTER(C.c_uint8)), ("valid", C.POINTER(C.c_uint8)),
                ("tile_col_off", C.POINTER(C.c_int32)), ("ew_nnz", C.c_int64),
                ("ew_col_ptr", C.POINTER(C.c_int32)), ("ew_row", C.POINTER(C.c_int32)),
                ("ew_val", C.POINTER(C.c_uint16)), ("dtype", C.c_int32)]


class LaunchOpts(C.Structure):
    """tw_launch_opts: per-call launch options (see include/twgemm.h)."""
    _fields_ = [("tile_m", C.c_int32), ("kernel", C.c_int32), ("depth", C.c_int32), ("waves", C.c_int32),
                ("ksplit", C.c_int32), ("xcd_map", C.c_int32), ("wg_split", C.c_int32), ("idx_route", C.c_int32), ("tiles_per_wg", C.c_int32),
                ("workspace_dev", C.c_void_p), ("workspace_bytes", C.c_size_t)]


def lib_path() -> str:
    """In-tree library; TWGEMM_LIB may point at another build of the same ABI."""
    return os.environ.get("TWGEMM_LIB") or os.path.join(
        os.path.dirname(os.path.abspath(__file__)), "libtwgemm.so")


def lib():
    global _lib
    if _lib is None:
        p = lib_path()
        if not os.path.exists(p):
            raise ImportError(f"{p} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        # PyTorch ships its own HIP/HSA runtime; it has to be the first one in the
        # process, or torch later finds no GPU.  libtwgemm.so then binds to it.
        import torch  # noqa: F401
        L = C.CDLL(p)
        vp, i = C.c_void_p, C.c_int
        L.tw_status_str.restype = C.c_char_p
        L.tw_status_str.argtypes = [i]
        L.tw_pack_host.argtypes = [vp, vp, vp, i, i, i, i, C.POINTER(vp)]
        L.tw_pack.argtypes = L.tw_pack_host.argtypes
        L.tw_upload.argtypes = [vp]
        L.tw_concat.argtypes = [C.POINTER(vp), i, i, C.POINTER(vp)]
        L.tw_prune_workspace_bytes.argtypes = [i, i, i, C.POINTER(C.c_size_t)]
        L.tw_prune_dev.argtypes = [vp, i, i, i, i, i, i, i, vp, vp, vp, C.c_size_t, vp]
        L.tw_prune_dev_static.argtypes = [vp, i, i, i, i, i, i, i, vp, vp, vp]
        L.tw_pack_dev.argtypes = [vp, i, vp, vp, i, i, i, i, vp, C.POINTER(vp)]
        L.tw_gemm.argtypes = [vp, i, i, i, vp, vp, i, vp]
        L.tw_pack_i8_host.argtypes = [vp, vp, vp, i, i, i, i, C.POINTER(vp)]
        L.tw_pack_i8.argtypes = L.tw_pack_i8_host.argtypes
        L.tw_gemm_i8.argtypes = [vp, i, i, vp, vp, i, i, C.c_float, vp]
        L.tw_dense_gemm_i8.argtypes = [vp, vp, vp, i, i, i, i, i, i, i, C.c_float, vp]
        L.tw_dense_gemm.argtypes = [vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.tw_conv_bind.argtypes = [vp, C.POINTER(_ConvGeom), C.c_int64, C.POINTER(C.c_void_p)]
        L.tw_conv_free.argtypes = [vp]
        L.tw_gemm_ex.argtypes = [vp, i, i, i, vp, vp, i, C.POINTER(LaunchOpts), vp]
        L.tw_launch_opts_init.argtypes = [C.POINTER(LaunchOpts)]
        L.tw_gemm_workspace_bytes.argtypes = [vp, i, C.POINTER(C.c_size_t)]
        L.tw_workspace_init.argtypes = [vp, C.c_size_t, vp]
        L.tw_conv_gemm.argtypes = [vp, vp, vp, i, vp]
        L.tw_conv_gemm_i8.argtypes = [vp, vp, vp, i, i, C.c_float, vp]
        L.tw_calibrate.argtypes = [i, vp, vp, C.c_size_t, i, vp, C.POINTER(C.c_double)]
        L.tw_export.argtypes = [vp, C.POINTER(_View)]
        L.tw_unpack.argtypes = [vp, vp, vp]
        L.tw_free.argtypes = [vp]
        L.tw_set_option.argtypes = [C.c_char_p, i]
        L.tw_flop_counts.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        for name in EXPORTED_SYMBOLS:
            if name != "tw_status_str":
                getattr(L, name).restype = i
        _lib = L
    return _lib


def _check(st: int, what: str):
    if st != 0:
        raise TwError(st, what)


def _host_ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class _ConvGeom(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("C", "R", "S", "B", "H", "W", "P", "L")]


class PackedWeight:
    """Owner of a tw_handle_t."""

    def __init__(self, handle: C.c_void_p):
        self._h = handle

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("handle already freed")
        return self._h

    def upload(self):
        _check(lib().tw_upload(self.handle), "tw_upload")
        return self

    def export(self) -> dict:
        """tw_export as numpy copies, in the layout of the logical packed form."""
        v = _View()
        _check(lib().tw_export(self.handle, C.byref(v)), "tw_export")
        nt, nk = v.n_tiles, v.n_kept

        def arr(ptr, n, dt):
            if n == 0 or not ptr:
                return np.zeros(0, dt)
            return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dt, copy=True)

        tko = arr(v.tile_k_off, nt + 1, np.int32) if nt >= 0 else np.zeros(1, np.int32)
        sk = int(tko[-1]) if tko.size else 0
        rows = arr(v.row_idx, sk, np.int32)
        ctok = arr(v.cto_k, sk, np.int32)
        voff = arr(v.val_off, nt + 1, np.int64)
        vals = arr(v.values, int(voff[-1]) if voff.size else 0, np.uint16)
        if v.dtype == DTYPE_I8:          # int8 values travel sign-extended to 16 bits
            vals = vals.view(np.int16).astype(np.int8)
        out = dict(K=v.K, N=v.N, G=v.G, pattern=v.pattern, dtype=v.dtype, n_kept=nk, n_tiles=nt,
                   col_idx=arr(v.col_idx, nk, np.int32), cto_n=arr(v.cto_n, nk, np.int32),
                   row_idx=[rows[tko[t]:tko[t + 1]] for t in range(nt)],
                   cto_k=[ctok[tko[t]:tko[t + 1]] for t in range(nt)])
        tco = arr(v.tile_col_off, nt + 1, np.int32)
        out["tile_col_off"] = tco
        widths = [int(tco[t + 1] - tco[t]) for t in range(nt)]
        if v.pattern in (PATTERN_TW, PATTERN_TEW):
            out["values"] = [vals[voff[t]:voff[t + 1]].reshape(int(tko[t + 1] - tko[t]), widths[t])
                             for t in range(nt)]
            if v.pattern == PATTERN_TEW:
                out["ew_col_ptr"] = arr(v.ew_col_ptr, v.N + 1, np.int32)
                out["ew_row"] = arr(v.ew_row, int(v.ew_nnz), np.int32)
                out["ew_val"] = arr(v.ew_val, int(v.ew_nnz), np.uint16)
        else:
            moff = arr(v.meta_off, nt + 1, np.int64)
            meta = arr(v.meta, int(moff[-1]) if moff.size else 0, np.uint8)
            valid = arr(v.valid, int(moff[-1]) if moff.size else 0, np.uint8)
            ng = [(int(tko[t + 1] - tko[t]) + 3) // 4 for t in range(nt)]
            out["values"] = [vals[voff[t]:voff[t + 1]].reshape(ng[t], 2, widths[t]) for t in range(nt)]
            out["meta"] = [meta[moff[t]:moff[t + 1]].reshape(ng[t], widths[t]) for t in range(nt)]
            out["valid"] = [valid[moff[t]:moff[t + 1]].reshape(ng[t], widths[t]) for t in range(nt)]
        return out

    def unpack(self):
        v = _View()
        _check(lib().tw_export(self.handle, C.byref(v)), "tw_export")
        Bm = np.empty((v.K, v.N), np.uint16)
        mask = np.empty((v.K, v.N), np.uint8)
        _check(lib().tw_unpack(self.handle, _host_ptr(Bm), _host_ptr(mask)), "tw_unpack")
        if v.dtype == DTYPE_I8:
            Bm = Bm.view(np.int16).astype(np.int8)
        return Bm, mask

    def flop_counts(self):
        """(sum K_t*W_t, sum K_t, rows of A kept by at least one tile)."""
        a, b, u = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib().tw_flop_counts(self.handle, C.byref(a), C.byref(b), C.byref(u)), "tw_flop_counts")
        return a.value, b.value, u.value

    def free(self):
        if self._h is not None:
            h, self._h = self._h, None
            _check(lib().tw_free(h), "tw_free")

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _pack(fn_name, B16, mask, G, pattern, tile_mask):
    B16 = np.ascontiguousarray(B16)
    if B16.dtype != np.float16 and B16.dtype != np.uint16:
        raise TypeError("B must be fp16 (or its uint16 bit patterns)")
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.shape != B16.shape or B16.ndim != 2:
        raise ValueError("B and mask must be K x N")
    if tile_mask is not None:
        tile_mask = np.ascontiguousarray(tile_mask, dtype=np.uint8)
        if tile_mask.shape != B16.shape:
            raise ValueError("tile_mask must be K x N")
    K, N = B16.shape
    h = C.c_void_p()
    st = getattr(lib(), fn_name)(_host_ptr(B16), _host_ptr(mask), _host_ptr(tile_mask),
                                 K, N, int(G), int(pattern), C.byref(h))
    _check(st, fn_name)
    return PackedWeight(h)


def tw_pack_host(B16, mask, G, pattern, tile_mask=None) -> PackedWeight:
    return _pack("tw_pack_host", B16, mask, G, pattern, tile_mask)


def tw_pack(B16, mask, G, pattern, tile_mask=None) -> PackedWeight:
    return _pack("tw_pack", B16, mask, G, pattern, tile_mask)


def _pack_i8(fn_name, B8, mask, G, pattern, tile_mask):
    B8 = np.ascontiguousarray(B8)
    if B8.dtype != np.int8:
        raise TypeError("B must be int8")
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.shape != B8.shape or B8.ndim != 2:
        raise ValueError("B and mask must be K x N")
    if tile_mask is not None:
        tile_mask = np.ascontiguousarray(tile_mask, dtype=np.uint8)
        if tile_mask.shape != B8.shape:
            raise ValueError("tile_mask must be K x N")
    K, N = B8.shape
    h = C.c_void_p()
    _check(getattr(lib(), fn_name)(_host_ptr(B8), _host_ptr(mask), _host_ptr(tile_mask), K, N, int(G),
                                   int(pattern), C.byref(h)), fn_name)
    return PackedWeight(h)


def tw_pack_i8_host(B8, mask, G, pattern=PATTERN_TW, tile_mask=None) -> PackedWeight:
    return _pack_i8("tw_pack_i8_host", B8, mask, G, pattern, tile_mask)


def tw_pack_i8(B8, mask, G, pattern=PATTERN_TW, tile_mask=None) -> PackedWeight:
    return _pack_i8("tw_pack_i8", B8, mask, G, pattern, tile_mask)


def tw_prune_workspace_bytes(K: int, N: int, G: int) -> int:
    n = C.c_size_t()
    _check(lib().tw_prune_workspace_bytes(K, N, G, C.byref(n)), "tw_prune_workspace_bytes")
    return n.value


def tw_prune_dev(B_ptr: int, K: int, N: int, ldb: int, G: int, pattern: int, n_cols_pruned: int,
                 rows_per_tile: int, mask_ptr: int, tile_mask_ptr, workspace_ptr: int, workspace_bytes: int,
                 stream: int = 0):
    """Device addresses in, K x N byte masks out (device); see include/twgemm.h."""
    _check(lib().tw_prune_dev(B_ptr, K, N, ldb, G, int(pattern), n_cols_pruned, rows_per_tile, mask_ptr,
                              tile_mask_ptr, workspace_ptr, workspace_bytes, stream), "tw_prune_dev")


def tw_prune_dev_static(B_ptr: int, K: int, N: int, ldb: int, G: int, pattern: int, n_cols_pruned: int,
                        rows_per_tile: int, mask_ptr: int, tile_mask_ptr, stream: int = 0):
    """tw_prune_dev without a workspace argument: the scratch is a fixed array inside the library."""
    _check(lib().tw_prune_dev_static(B_ptr, K, N, ldb, G, int(pattern), n_cols_pruned, rows_per_tile, mask_ptr,
                                     tile_mask_ptr, stream), "tw_prune_dev_static")


def tw_pack_dev(B_ptr: int, ldb: int, mask_ptr: int, tile_mask_ptr, K: int, N: int, G: int, pattern: int,
                stream: int = 0) -> PackedWeight:
    h = C.c_void_p()
    _check(lib().tw_pack_dev(B_ptr, ldb, mask_ptr, tile_mask_ptr, K, N, int(G), int(pattern), stream, C.byref(h)),
           "tw_pack_dev")
    return PackedWeight(h)


def tw_concat(parts, upload: bool = True) -> PackedWeight:
    """One handle for the packed weights `parts` side by side along N."""
    arr = (C.c_void_p * len(parts))(*[p.handle for p in parts])
    h = C.c_void_p()
    _check(lib().tw_concat(arr, len(parts), int(bool(upload)), C.byref(h)), "tw_concat")
    return PackedWeight(h)


def tw_gemm(A_ptr: int, M: int, lda: int, layout: int, packed: PackedWeight, C_ptr: int,
            ldc: int, stream: int = 0):
    """A_ptr / C_ptr: device addresses (e.g. torch.Tensor.data_ptr()), stream: hipStream_t."""
    _check(lib().tw_gemm(A_ptr, M, lda, layout, packed.handle, C_ptr, ldc, stream), "tw_gemm")


def tw_dense_gemm(A_ptr: int, B_ptr: int, C_ptr: int, M: int, K: int, N: int, lda: int,
                  ldb: int, ldc: int, layout: int, stream: int = 0):
    _check(lib().tw_dense_gemm(A_ptr, B_ptr, C_ptr, M, K, N, lda, ldb, ldc, layout, stream),
           "tw_dense_gemm")


def tw_gemm_i8(A_ptr: int, M: int, lda: int, packed: PackedWeight, C_ptr: int, ldc: int,
               c_dtype: int = 0, scale: float = 1.0, stream: int = 0):
    """int8 A (K x M) times a packed int8 weight; C (N x M) int32 (c_dtype 0) or requantised int8 (1)."""
    _check(lib().tw_gemm_i8(A_ptr, M, lda, packed.handle, C_ptr, ldc, c_dtype, scale, stream), "tw_gemm_i8")


def tw_dense_gemm_i8(A_ptr: int, B_ptr: int, C_ptr: int, M: int, K: int, N: int, lda: int, ldb: int,
                     ldc: int, c_dtype: int = 0, scale: float = 1.0, stream: int = 0):
    _check(lib().tw_dense_gemm_i8(A_ptr, B_ptr, C_ptr, M, K, N, lda, ldb, ldc, c_dtype, scale, stream),
           "tw_dense_gemm_i8")


class ConvBinding:
    """Owner of a tw_conv_t; keeps its packed weight alive."""

    def __init__(self, handle, packed):
        self._b, self._packed = handle, packed

    @property
    def handle(self):
        if self._b is None:
            raise ValueError("binding already freed")
        return self._b

    def free(self):
        if self._b is not None:
            b, self._b = self._b, None
            _check(lib().tw_conv_free(b), "tw_conv_free")

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def tw_conv_bind(packed: PackedWeight, geom, ldx: int) -> ConvBinding:
    """geom: anything with integer attributes C, R, S, B, H, W, P, L (see tw_conv_geom)."""
    g = _ConvGeom(*(int(getattr(geom, n)) for n in ("C", "R", "S", "B", "H", "W", "P", "L")))
    b = C.c_void_p()
    _check(lib().tw_conv_bind(packed.handle, C.byref(g), int(ldx), C.byref(b)), "tw_conv_bind")
    return ConvBinding(b, packed)


def tw_conv_gemm(X_ptr: int, binding: ConvBinding, C_ptr: int, ldc: int, stream: int = 0):
    _check(lib().tw_conv_gemm(X_ptr, binding.handle, C_ptr, ldc, stream), "tw_conv_gemm")


def tw_conv_gemm_i8(X_ptr: int, binding: ConvBinding, C_ptr: int, ldc: int, c_dtype: int = 0, scale: float = 1.0,
                    stream: int = 0):
    _check(lib().tw_conv_gemm_i8(X_ptr, binding.handle, C_ptr, ldc, c_dtype, scale, stream), "tw_conv_gemm_i8")


def tw_launch_opts(**kw) -> LaunchOpts:
    """The default launch options with the given fields replaced."""
    o = LaunchOpts()
    _check(lib().tw_launch_opts_init(C.byref(o)), "tw_launch_opts_init")
    for k, v in kw.items():
        if not hasattr(o, k):
            raise TypeError(f"tw_launch_opts has no field {k!r}")
        setattr(o, k, v)
    return o


def tw_gemm_workspace_bytes(packed: PackedWeight, M: int) -> int:
    n = C.c_size_t()
    _check(lib().tw_gemm_workspace_bytes(packed.handle, M, C.byref(n)), "tw_gemm_workspace_bytes")
    return n.value


def tw_workspace_init(ws_ptr: int, ws_bytes: int, stream: int = 0):
    _check(lib().tw_workspace_init(ws_ptr, ws_bytes, stream), "tw_workspace_init")


def tw_gemm_ex(A_ptr: int, M: int, lda: int, layout: int, packed: PackedWeight, C_ptr: int, ldc: int,
               opts: LaunchOpts | None = None, stream: int = 0):
    _check(lib().tw_gemm_ex(A_ptr, M, lda, layout, packed.handle, C_ptr, ldc,
                            C.byref(opts) if opts is not None else None, stream), "tw_gemm_ex")


CAL_COPY, CAL_READ, CAL_WRITE, CAL_STORE_CT, CAL_MFMA_F16, CAL_SMFMAC_F16, CAL_MFMA_I8 = 0, 1, 2, 3, 10, 11, 12


def tw_calibrate(kind: int, dst_ptr: int, src_ptr, nbytes: int, iters: int = 0, stream: int = 0) -> float:
    """Enqueues one streaming / matrix-core-loop kernel; returns the work of the launch
    (bytes or dense-equivalent operations)."""
    units = C.c_double()
    _check(lib().tw_calibrate(kind, dst_ptr, src_ptr, nbytes, iters, stream, C.byref(units)), "tw_calibrate")
    return units.value


def tw_set_option(name: str, value: int):
    _check(lib().tw_set_option(name.encode(), int(value)), "tw_set_option")
