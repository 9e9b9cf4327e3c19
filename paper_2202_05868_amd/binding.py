"""ctypes binding of ``libvbr_spmm.so`` (see ``include/vbr_spmm.h``).

Argument marshalling only: every step of the path runs inside the library.  PyTorch is used for
device memory and the current HIP stream, nothing else.  There is no fallback: if the library is
not built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("VBR_SPMM_LIB") or os.path.join(_HERE, "libvbr_spmm.so")   # the built library; the variable names another build of it

VBR_F16, VBR_BF16 = 0, 1
_DTYPES = {"f16": VBR_F16, "bf16": VBR_BF16}

EXPORTS = ("sa1_reorder", "vbr_build", "vbr_get_index", "vbr_unpack_block", "vbr_device_bytes",
           "vbr_upload", "vbr_spmm", "vbr_get_schedule", "vbr_free", "vbr_strerror",
           "vbr_last_hip_error", "sa1_blocking_curve", "csr_spmm_create", "csr_device_bytes", "csr_upload",
           "csr_spmm", "csr_free", "vbr_probe_launch", "vbr_get_launches", "vbr_audit", "vbr_get_tile_ksteps")


class VbrError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        msg = _lib.vbr_strerror(code).decode()
        if code == -3:
            msg += " (hipError %d)" % _lib.vbr_last_hip_error()
        super().__init__("%s: %s" % (what, msg))


class _Csr(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("n_cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("vals", ctypes.c_void_p),
                ("dtype", ctypes.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: run `python -m paper_2202_05868_amd.build` (hipcc, gfx950); "
                          "there is no CPU fallback" % LIB_PATH)
    # PyTorch ships its own HIP runtime under the same soname as the system one; it has to be the
    # first in the process, or the two get mixed and no device is found.  Importing torch first
    # makes the library bind to the runtime torch's streams and allocations live in.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    P = ctypes.POINTER
    lib.sa1_reorder.argtypes = [P(_Csr), i32, dbl, vp, vp, P(i32)]
    lib.vbr_build.argtypes = [P(_Csr), vp, vp, i32, i32, P(vp)]
    lib.vbr_get_index.argtypes = [vp, P(vp), P(vp), P(vp), P(vp), P(vp), P(i64), P(i64), P(i64)]
    lib.vbr_unpack_block.argtypes = [vp, i64, vp]
    lib.vbr_device_bytes.argtypes = [vp]
    lib.vbr_device_bytes.restype = i64
    lib.vbr_upload.argtypes = [vp, vp, vp]
    lib.vbr_spmm.argtypes = [vp, vp, i64, vp, i64, i64, vp]
    lib.vbr_get_schedule.argtypes = [vp, P(i64), P(i64), P(i64)]
    lib.vbr_get_launches.argtypes = [vp, i64, P(i32), vp, vp, vp]
    lib.vbr_get_launches.restype = ctypes.c_int
    lib.vbr_get_tile_ksteps.argtypes = [vp, vp, i64]
    lib.vbr_get_tile_ksteps.restype = i64
    lib.vbr_audit.argtypes = [vp]
    lib.vbr_audit.restype = ctypes.c_int
    lib.vbr_free.argtypes = [vp]
    lib.vbr_free.restype = None
    lib.vbr_strerror.argtypes = [ctypes.c_int]
    lib.vbr_strerror.restype = ctypes.c_char_p
    lib.vbr_last_hip_error.restype = ctypes.c_int
    lib.sa1_blocking_curve.argtypes = [P(_Csr), i32, vp, i32, i64, vp, vp, vp, vp, P(i32)]
    lib.csr_spmm_create.argtypes = [P(_Csr), P(vp)]
    lib.csr_device_bytes.argtypes = [vp]
    lib.csr_device_bytes.restype = i64
    lib.csr_upload.argtypes = [vp, vp, vp]
    lib.csr_spmm.argtypes = [vp, vp, i64, vp, i64, i64, vp]
    lib.csr_free.argtypes = [vp]
    lib.csr_free.restype = None
    lib.vbr_probe_launch.argtypes = [i32, vp, i64, i32, vp, P(dbl)]
    lib.vbr_probe_launch.restype = ctypes.c_int
    for name in ("sa1_reorder", "vbr_build", "vbr_get_index", "vbr_unpack_block", "vbr_upload",
                 "vbr_spmm", "vbr_get_schedule", "sa1_blocking_curve", "csr_spmm_create", "csr_upload", "csr_spmm"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None and a.size else None


def _csr_struct(csr: dict, need_vals: bool):
    """Marshal a CSR dict (see synth.py) into the C struct; returns (struct, keepalive)."""
    row_ptr = np.ascontiguousarray(csr["row_ptr"], dtype=np.int64)
    col_idx = np.ascontiguousarray(csr["col_idx"], dtype=np.int32)
    vals = np.ascontiguousarray(csr["vals"], dtype=np.uint16) if (need_vals or csr.get("vals") is not None) else None
    s = _Csr(int(csr["n_rows"]), int(csr["n_cols"]), int(csr["nnz"]),
             row_ptr.ctypes.data_as(ctypes.c_void_p), _ptr(col_idx), _ptr(vals), _DTYPES[csr["dtype"]])
    return s, (row_ptr, col_idx, vals)


def sa1_reorder(csr: dict, col_block: int, tau: float):
    """1-SA row reordering.  Returns (perm int32[n_rows], row_groups int32[G+1])."""
    s, keep = _csr_struct(csr, need_vals=False)
    m = int(csr["n_rows"])
    perm = np.empty(m, dtype=np.int32)
    rg = np.empty(m + 1, dtype=np.int32)
    ng = ctypes.c_int32(0)
    rc = _lib.sa1_reorder(ctypes.byref(s), int(col_block), float(tau), perm.ctypes.data_as(ctypes.c_void_p),
                          rg.ctypes.data_as(ctypes.c_void_p), ctypes.byref(ng))
    if rc != 0:
        raise VbrError(rc, "sa1_reorder")
    return perm, rg[: ng.value + 1].copy()


def _check_operands(what: str, dtype: str, n_rows: int, n_cols: int, dev_buf, b, c):
    """Everything about B and C that the C ABI cannot see (it gets raw addresses): types, shapes,
    strides and the device they live on.  A short B or C would be read or written out of bounds on
    the device, so nothing is launched unless these hold.  Returns C (allocated here if None)."""
    import torch
    want = torch.float16 if dtype == "f16" else torch.bfloat16
    if b.dtype != want or b.dim() != 2 or (b.shape[1] > 1 and b.stride(1) != 1):
        raise ValueError("%s: B must be a 2-D %s tensor with unit column stride" % (what, want))
    if b.shape[0] < n_cols:
        raise ValueError("%s: B has %d rows, the matrix has %d columns" % (what, b.shape[0], n_cols))
    n = b.shape[1]
    if c is None:
        c = torch.empty((n_rows, n), dtype=torch.float32, device=b.device)
    if c.dtype != torch.float32 or c.dim() != 2 or tuple(c.shape) != (n_rows, n) or (n > 1 and c.stride(1) != 1):
        raise ValueError("%s: C must be a 2-D float32 tensor of shape (%d, %d) with unit column stride" % (what, n_rows, n))
    if (n_rows > 1 and c.stride(0) < n) or (b.shape[0] > 1 and b.stride(0) < n):
        raise ValueError("%s: rows of B and C must not overlap (row stride >= N)" % what)
    if dev_buf is None:
        raise VbrError(-4, what)
    if b.device != dev_buf.device or c.device != dev_buf.device:
        raise ValueError("%s: B and C must be on %s, where the matrix was uploaded" % (what, dev_buf.device))
    return c


class Vbr:
    """Owner of a ``vbr_t`` handle (and, after ``upload``, of the torch tensor behind it)."""

    def __init__(self, handle, dtype: str, n_rows: int, n_cols: int):
        self._h = ctypes.c_void_p(handle)
        self.dtype = dtype
        self.n_rows = int(n_rows)
        self.n_cols = int(n_cols)
        self._dev = None

    def close(self):
        if self._h:
            _lib.vbr_free(self._h)
            self._h = ctypes.c_void_p(None)
            self._dev = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- index views (copied out)
    def index(self) -> dict:
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        rg, pm, bp, bc, bo = vp(), vp(), vp(), vp(), vp()
        ng, nb, se = i64(), i64(), i64()
        rc = _lib.vbr_get_index(self._h, ctypes.byref(rg), ctypes.byref(pm), ctypes.byref(bp), ctypes.byref(bc),
                                ctypes.byref(bo), ctypes.byref(ng), ctypes.byref(nb), ctypes.byref(se))
        if rc != 0:
            raise VbrError(rc, "vbr_get_index")

        def view(p, n, ct, dt):
            if n == 0 or not p.value:
                return np.zeros(0, dtype=dt)
            return np.ctypeslib.as_array(ctypes.cast(p, ctypes.POINTER(ct)), shape=(n,)).astype(dt, copy=True)

        g, b = ng.value, nb.value
        row_groups = view(rg, g + 1, ctypes.c_int32, np.int32)
        n_rows = int(row_groups[-1]) if g + 1 > 0 and row_groups.size else 0
        return dict(row_groups=row_groups, perm=view(pm, n_rows, ctypes.c_int32, np.int32),
                    blk_ptr=view(bp, g + 1, ctypes.c_int64, np.int64), blk_col=view(bc, b, ctypes.c_int32, np.int32),
                    blk_off=view(bo, b + 1, ctypes.c_int64, np.int64), n_groups=g, n_blocks=b,
                    stored_elems=se.value)

    def schedule(self) -> dict:
        i64 = ctypes.c_int64
        a, b, c = i64(), i64(), i64()
        rc = _lib.vbr_get_schedule(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
        if rc != 0:
            raise VbrError(rc, "vbr_get_schedule")
        return dict(n_tiles=a.value, n_ksteps=b.value, packed_elems=c.value)

    LAUNCH_KINDS = ("vbr_spmm_panel_kernel", "vbr_spmm_kernel<1 slab>", "vbr_spmm_kernel<2 slabs>",
                    "vbr_spmm_kernel<4 slabs>", "vbr_spmm_kernel<8 slabs>", "vbr_spmm_mixed_kernel",
                    "vbr_spmm_kernel<1 slab, column-gathered>", "vbr_spmm_kernel<2 slabs, column-gathered>",
                    "vbr_spmm_kernel<4 slabs, column-gathered>", "vbr_spmm_kernel<8 slabs, column-gathered>")

    def launches(self, n: int) -> list:
        """The kernel launches one ``spmm`` with dense width ``n`` issues, from the library's plan."""
        kinds = np.zeros(16, dtype=np.int32)
        tiles = np.zeros(16, dtype=np.int64)
        wgs = np.zeros(16, dtype=np.int64)
        cnt = ctypes.c_int32(0)
        rc = _lib.vbr_get_launches(self._h, int(n), ctypes.byref(cnt), kinds.ctypes.data_as(ctypes.c_void_p),
                                   tiles.ctypes.data_as(ctypes.c_void_p), wgs.ctypes.data_as(ctypes.c_void_p))
        if rc != 0:
            raise VbrError(rc, "vbr_get_launches")
        return [dict(kernel=self.LAUNCH_KINDS[int(kinds[i])], tiles=int(tiles[i]), workgroups=int(wgs[i]))
                for i in range(cnt.value)]

    def unpack_block(self, blk: int, h: int, col_block: int) -> np.ndarray:
        out = np.empty((h, col_block), dtype=np.uint16)
        rc = _lib.vbr_unpack_block(self._h, int(blk), out.ctypes.data_as(ctypes.c_void_p))
        if rc != 0:
            raise VbrError(rc, "vbr_unpack_block")
        return out

    def tile_ksteps(self) -> np.ndarray:
        """K-steps of every workgroup tile of the schedule (tiles, column-gathered slabs, panels)."""
        n = int(_lib.vbr_get_tile_ksteps(self._h, None, 0))
        out = np.zeros(max(n, 1), dtype=np.int64)
        _lib.vbr_get_tile_ksteps(self._h, out.ctypes.data_as(ctypes.c_void_p), n)
        return out[:n]

    def audit(self) -> None:
        """Raise unless every index the kernels use lies inside what it indexes."""
        rc = _lib.vbr_audit(self._h)
        if rc != 0:
            raise VbrError(rc, "vbr_audit")

    def device_bytes(self) -> int:
        return int(_lib.vbr_device_bytes(self._h))

    # ---- GPU side
    def upload(self, device="cuda:0"):
        import torch
        buf = torch.empty(self.device_bytes(), dtype=torch.uint8, device=device)
        assert buf.data_ptr() % 256 == 0
        with torch.cuda.device(buf.device):
            stream = torch.cuda.current_stream().cuda_stream
            rc = _lib.vbr_upload(self._h, ctypes.c_void_p(buf.data_ptr()), ctypes.c_void_p(stream))
        if rc != 0:
            raise VbrError(rc, "vbr_upload")
        self._dev = buf
        return self

    def spmm(self, b, c=None):
        """C = A.B.  ``b``: torch [K, N] float16/bfloat16 on the GPU of the uploaded matrix, K >= the
        matrix's columns (row stride free, unit column stride); ``c``: optional torch [M, N] float32
        output on the same GPU.  Runs on torch's current stream."""
        import torch
        c = _check_operands("vbr_spmm", self.dtype, self.n_rows, self.n_cols, self._dev, b, c)
        n = b.shape[1]
        with torch.cuda.device(b.device):
            stream = torch.cuda.current_stream().cuda_stream
            rc = vbr_spmm_raw(self, b.data_ptr(), b.stride(0), c.data_ptr(), c.stride(0), n, stream)
        if rc != 0:
            raise VbrError(rc, "vbr_spmm")
        return c


def vbr_spmm_raw(v: Vbr, b_ptr: int, ldb: int, c_ptr: int, ldc: int, n: int, stream: int) -> int:
    """The C call itself, on raw device addresses; returns the library's code."""
    return int(_lib.vbr_spmm(v._h, ctypes.c_void_p(b_ptr), int(ldb), ctypes.c_void_p(c_ptr), int(ldc), int(n),
                             ctypes.c_void_p(stream)))


def vbr_build(csr: dict, perm: np.ndarray, row_groups: np.ndarray, col_block: int) -> Vbr:
    s, keep = _csr_struct(csr, need_vals=True)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    row_groups = np.ascontiguousarray(row_groups, dtype=np.int32)
    h = ctypes.c_void_p()
    rc = _lib.vbr_build(ctypes.byref(s), perm.ctypes.data_as(ctypes.c_void_p),
                        row_groups.ctypes.data_as(ctypes.c_void_p), int(row_groups.size - 1), int(col_block),
                        ctypes.byref(h))
    if rc != 0:
        raise VbrError(rc, "vbr_build")
    return Vbr(h.value, csr["dtype"], csr["n_rows"], csr["n_cols"])


def vbr_spmm(v: Vbr, b, c=None):
    return v.spmm(b, c)


def sa1_blocking_curve(csr: dict, col_block: int, taus, target_height: int) -> dict:
    """Blocking curve of 1-SA over the thresholds ``taus`` and the blocking selected by the rule
    "average block height nearest to ``target_height``".  Returns the library's integer counts per
    threshold and ``selected`` (index into ``taus``)."""
    s, keep = _csr_struct(csr, need_vals=False)
    t = np.ascontiguousarray(taus, dtype=np.float64)
    out = {k: np.zeros(t.size, dtype=np.int64) for k in ("n_groups", "n_blocks", "stored_elems", "sum_heights")}
    sel = ctypes.c_int32(0)
    rc = _lib.sa1_blocking_curve(ctypes.byref(s), int(col_block), t.ctypes.data_as(ctypes.c_void_p), int(t.size),
                                 int(target_height), *[out[k].ctypes.data_as(ctypes.c_void_p) for k in
                                                       ("n_groups", "n_blocks", "stored_elems", "sum_heights")],
                                 ctypes.byref(sel))
    if rc != 0:
        raise VbrError(rc, "sa1_blocking_curve")
    out["selected"] = int(sel.value)
    out["taus"] = t
    return out


class CsrDev:
    """Owner of a ``csr_dev_t`` handle: the CSR matrix on the GPU for the comparator kernel."""

    def __init__(self, csr: dict):
        s, keep = _csr_struct(csr, need_vals=True)
        h = ctypes.c_void_p()
        rc = _lib.csr_spmm_create(ctypes.byref(s), ctypes.byref(h))
        if rc != 0:
            raise VbrError(rc, "csr_spmm_create")
        self._h = h
        self.dtype = csr["dtype"]
        self.n_rows = int(csr["n_rows"])
        self.n_cols = int(csr["n_cols"])
        self._dev = None

    def close(self):
        if self._h:
            _lib.csr_free(self._h)
            self._h = ctypes.c_void_p(None)
            self._dev = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def upload(self, device="cuda:0"):
        import torch
        buf = torch.empty(int(_lib.csr_device_bytes(self._h)), dtype=torch.uint8, device=device)
        assert buf.data_ptr() % 256 == 0
        with torch.cuda.device(buf.device):
            stream = torch.cuda.current_stream().cuda_stream
            rc = _lib.csr_upload(self._h, ctypes.c_void_p(buf.data_ptr()), ctypes.c_void_p(stream))
        if rc != 0:
            raise VbrError(rc, "csr_upload")
        self._dev = buf
        return self

    def spmm(self, b, c=None):
        import torch
        c = _check_operands("csr_spmm", self.dtype, self.n_rows, self.n_cols, self._dev, b, c)
        n = b.shape[1]
        with torch.cuda.device(b.device):
            stream = torch.cuda.current_stream().cuda_stream
            rc = int(_lib.csr_spmm(self._h, ctypes.c_void_p(b.data_ptr()), int(b.stride(0)), ctypes.c_void_p(c.data_ptr()),
                                   int(c.stride(0)), int(n), ctypes.c_void_p(stream)))
        if rc != 0:
            raise VbrError(rc, "csr_spmm")
        return c


PROBES = {"mfma_16x16x32_f16": 0, "mfma_16x16x16_f16": 1, "mfma_32x32x16_f16": 2, "lds_read_tr_b64": 3,
          "lds_read_b64": 4, "lds_read_b128": 5, "lds_dma_b128": 6, "hbm_copy": 7}


def vbr_probe_launch(kind: str, buf, iters: int) -> float:
    """Enqueue one launch of a denominator loop on torch's current stream; returns the work (flops
    or bytes) the launch performs.  ``buf``: a torch uint8 tensor on the GPU (caller-allocated)."""
    import torch
    work = ctypes.c_double(0.0)
    with torch.cuda.device(buf.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = int(_lib.vbr_probe_launch(PROBES[kind], ctypes.c_void_p(buf.data_ptr()), int(buf.numel()), int(iters),
                                       ctypes.c_void_p(stream), ctypes.byref(work)))
    if rc != 0:
        raise VbrError(rc, "vbr_probe_launch")
    return work.value
