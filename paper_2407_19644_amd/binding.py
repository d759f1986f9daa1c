"""ctypes binding of include/ubp.h: same names, argument marshalling only.

The library is loaded from the package directory (libubp.so, built by build.py).  If it is
missing the import of any entry point fails loudly; there is no fallback path.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libubp.so")

UBP_OK = 0
UBP_HOST_ONLY = -1
HOST_ONLY = UBP_HOST_ONLY


def layout_slot(sub_stripes, col_tiles):
    """Index of a (stripes per wavefront, column tiles per wavefront) layout in ubp_packed_info's 100+ / 200+ ... ranges."""
    return {1: 0, 2: 1, 4: 2}[sub_stripes] * 3 + {2: 0, 4: 1, 8: 2}[col_tiles]
DTYPES = {"f32": 0, "f16": 1, "bf16": 2}
_NP_OF = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}
EXPORTS = ("ubp_target_block_count", "ubp_select_reference", "ubp_pack", "ubp_packed_indptr",
           "ubp_packed_indices", "ubp_packed_values", "ubp_spmm", "ubp_spmm_plan", "ubp_packed_info",
           "ubp_packed_free", "ubp_status_string", "ubp_packed_device_error", "ubp_packed_layout",
           "ubp_spmm_prepare", "ubp_launch_floor", "ubp_block_scores", "ubp_select_greedy", "ubp_select_bed",
           "ubp_select_optimal", "ubp_selection_to_blocks", "ubp_select_blocks", "ubp_selection_efficacy",
           "ubp_spmm_fused")
ACTIVATIONS = {None: 0, "none": 0, "relu": 1, "clamp": 2}
SELECT_METHODS = {"greedy": 0, "bed": 1, "optimal": 2}


class UBPError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__("%s: %s (status %d)" % (where, status_string(code), code))


class Plan(ctypes.Structure):
    """Mirror of ubp_plan; zero fields mean 'choose automatically'."""
    _fields_ = [("kernel", ctypes.c_int32), ("sub_stripes", ctypes.c_int32), ("col_tiles", ctypes.c_int32),
                ("waves", ctypes.c_int32), ("rows_per_range", ctypes.c_int32), ("producers", ctypes.c_int32),
                ("wg_rows", ctypes.c_int32)]


class Epilogue(ctypes.Structure):
    """Mirror of ubp_epilogue."""
    _fields_ = [("bias_dev", ctypes.c_void_p), ("activation", ctypes.c_int32), ("lo", ctypes.c_float), ("hi", ctypes.c_float)]


_lib = None


def library_path():
    return _LIB_PATH


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("native library %s is missing: run `python -m paper_2407_19644_amd.build` "
                          "(there is no fallback implementation)" % _LIB_PATH)
    L = ctypes.CDLL(_LIB_PATH)
    i32, i64, u64, dbl, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p
    pi64 = ctypes.POINTER(i64)
    L.ubp_target_block_count.argtypes = [i32, i32, i32, i32, dbl]
    L.ubp_target_block_count.restype = i64
    L.ubp_select_reference.argtypes = [i32, i32, i32, i32, dbl, u64, i32, dbl, vp, i64, pi64]
    L.ubp_select_reference.restype = ctypes.c_int
    L.ubp_pack.argtypes = [vp, ctypes.c_int, i32, i32, i64, i32, i32, vp, i64, i32, ctypes.POINTER(vp)]
    L.ubp_pack.restype = ctypes.c_int
    for f in (L.ubp_packed_indptr, L.ubp_packed_indices, L.ubp_packed_values):
        f.argtypes = [vp, pi64]
        f.restype = vp
    L.ubp_spmm.argtypes = [vp, vp, i64, i32, vp, i64, ctypes.c_int, vp]
    L.ubp_spmm.restype = ctypes.c_int
    L.ubp_spmm_plan.argtypes = [vp, vp, i64, i32, vp, i64, ctypes.c_int, vp, ctypes.POINTER(Plan)]
    L.ubp_spmm_plan.restype = ctypes.c_int
    L.ubp_packed_info.argtypes = [vp, i32]
    L.ubp_packed_info.restype = i64
    L.ubp_packed_device_error.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32)]
    L.ubp_packed_device_error.restype = ctypes.c_int
    L.ubp_packed_layout.argtypes = [vp, i32, i32, i32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(vp),
                                    ctypes.POINTER(vp), ctypes.POINTER(vp), pi64, ctypes.POINTER(vp), pi64]
    L.ubp_packed_layout.restype = ctypes.c_int
    L.ubp_spmm_prepare.argtypes = [vp, vp, i64, i32, vp, i64, ctypes.c_int, ctypes.POINTER(Plan), ctypes.POINTER(Plan)]
    L.ubp_spmm_prepare.restype = ctypes.c_int
    L.ubp_spmm_fused.argtypes = [vp, vp, i64, i32, vp, i64, ctypes.c_int, ctypes.POINTER(Epilogue), vp, ctypes.POINTER(Plan)]
    L.ubp_spmm_fused.restype = ctypes.c_int
    L.ubp_launch_floor.argtypes = [vp]
    L.ubp_launch_floor.restype = ctypes.c_int
    L.ubp_block_scores.argtypes = [vp, ctypes.c_int, i64, i32, i32, i32, i32, i32, vp, i64]
    L.ubp_block_scores.restype = ctypes.c_int
    for f in (L.ubp_select_greedy, L.ubp_select_bed, L.ubp_select_optimal):
        f.argtypes = [vp, i64, i32, i64, vp, pi64]
        f.restype = ctypes.c_int
    L.ubp_selection_to_blocks.argtypes = [vp, i64, i32, i32, vp]
    L.ubp_selection_to_blocks.restype = ctypes.c_int
    L.ubp_select_blocks.argtypes = [vp, ctypes.c_int, i64, i32, i32, i32, i32, dbl, i32, i32, vp, i64, pi64]
    L.ubp_select_blocks.restype = ctypes.c_int
    L.ubp_selection_efficacy.argtypes = [vp, ctypes.c_int, i64, i32, i32, i32, i32, vp, i64, vp, i64, vp,
                                         ctypes.POINTER(dbl)]
    L.ubp_selection_efficacy.restype = ctypes.c_int
    L.ubp_packed_free.argtypes = [vp]
    L.ubp_packed_free.restype = None
    L.ubp_status_string.argtypes = [ctypes.c_int]
    L.ubp_status_string.restype = ctypes.c_char_p
    _lib = L
    return L


def status_string(code):
    return load_library().ubp_status_string(int(code)).decode()


def target_block_count(M, K, bh, bw, density):
    return int(load_library().ubp_target_block_count(M, K, bh, bw, float(density)))


def select_reference(M, K, bh, bw, density, seed, mode=0, zipf_s=0.0):
    """ubp_select_reference -> int32 array [nb, 2] of (r, c), sorted."""
    L = load_library()
    nb = ctypes.c_int64(0)
    need = L.ubp_target_block_count(M, K, bh, bw, float(density))
    if need < 0:
        raise UBPError(1, "ubp_select_reference")
    out = np.zeros((max(int(need), 1), 2), dtype=np.int32)
    rc = L.ubp_select_reference(M, K, bh, bw, float(density), int(seed), int(mode), float(zipf_s),
                                out.ctypes.data, int(need), ctypes.byref(nb))
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_select_reference")
    return out[:nb.value].copy()


def _weights(W_host, dtype):
    W = np.asarray(W_host)
    if W.ndim != 2 or W.dtype != _NP_OF[dtype] or W.strides[1] != W.itemsize or W.strides[0] % W.itemsize:
        raise ValueError("W must be a row-major 2-D array of %s" % _NP_OF[dtype].__name__)
    return W


def block_scores(W_host, dtype, bh, bw, aligned=False):
    """ubp_block_scores -> float64 array of b = M * (K // bw) scores, candidate k = i + M * j."""
    W = _weights(W_host, dtype)
    S = np.empty(W.shape[0] * (W.shape[1] // bw), dtype=np.float64)
    rc = load_library().ubp_block_scores(W.ctypes.data, DTYPES[dtype], W.strides[0] // W.itemsize, W.shape[0],
                                         W.shape[1], bh, bw, int(bool(aligned)), S.ctypes.data, S.size)
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_block_scores")
    return S


def _select(name, S, N, m):
    S = np.ascontiguousarray(S, dtype=np.float64)
    I = np.zeros(max(int(m), 1), dtype=np.int64)
    count = ctypes.c_int64(0)
    rc = getattr(load_library(), name)(S.ctypes.data, S.size, int(N), int(m), I.ctypes.data, ctypes.byref(count))
    if rc != UBP_OK:
        raise UBPError(rc, name)
    return I[:count.value].copy()


def select_greedy(S, N, m):
    """ubp_select_greedy -> int64 candidate indices in order of selection."""
    return _select("ubp_select_greedy", S, N, m)


def select_bed(S, N, m):
    """ubp_select_bed -> int64 candidate indices, ascending."""
    return _select("ubp_select_bed", S, N, m)


def select_optimal(S, N, m):
    """ubp_select_optimal -> int64 candidate indices, ascending; UBPError(5) if no m blocks fit."""
    return _select("ubp_select_optimal", S, N, m)


def selection_to_blocks(I, M, bw):
    """ubp_selection_to_blocks -> int32 array [count, 2] of (r, c)."""
    I = np.ascontiguousarray(I, dtype=np.int64)
    out = np.zeros((max(I.size, 1), 2), dtype=np.int32)
    rc = load_library().ubp_selection_to_blocks(I.ctypes.data, I.size, int(M), int(bw), out.ctypes.data)
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_selection_to_blocks")
    return out[:I.size].copy()


def select_blocks(W_host, dtype, bh, bw, density, method="bed", aligned=False):
    """ubp_select_blocks -> int32 array [nb, 2] of (r, c)."""
    W = _weights(W_host, dtype)
    L = load_library()
    need = L.ubp_target_block_count(W.shape[0], W.shape[1], bh, bw, float(density))
    if need < 0:
        raise UBPError(1, "ubp_select_blocks")
    out = np.zeros((max(int(need), 1), 2), dtype=np.int32)
    nb = ctypes.c_int64(0)
    rc = L.ubp_select_blocks(W.ctypes.data, DTYPES[dtype], W.strides[0] // W.itemsize, W.shape[0], W.shape[1], bh, bw,
                             float(density), SELECT_METHODS[method], int(bool(aligned)), out.ctypes.data, int(need),
                             ctypes.byref(nb))
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_select_blocks")
    return out[:nb.value].copy()


def selection_efficacy(W_host, dtype, bh, bw, ubp_blocks, abp_blocks):
    """ubp_selection_efficacy -> (efficacy, (l1_ubp, l1_abp, l1_ep))."""
    W = _weights(W_host, dtype)
    u = np.ascontiguousarray(np.asarray(ubp_blocks, dtype=np.int32).reshape(-1, 2))
    a = np.ascontiguousarray(np.asarray(abp_blocks, dtype=np.int32).reshape(-1, 2))
    l1 = np.zeros(3, dtype=np.float64)
    eff = ctypes.c_double(0.0)
    rc = load_library().ubp_selection_efficacy(W.ctypes.data, DTYPES[dtype], W.strides[0] // W.itemsize, W.shape[0],
                                               W.shape[1], bh, bw, u.ctypes.data, u.shape[0], a.ctypes.data, a.shape[0],
                                               l1.ctypes.data, ctypes.byref(eff))
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_selection_efficacy")
    return eff.value, tuple(l1.tolist())


class Packed:
    """Owner of a ubp_packed handle."""

    def __init__(self, handle, dtype):
        self._h = ctypes.c_void_p(handle)
        self.dtype = dtype

    @property
    def handle(self):
        if not self._h:
            raise ValueError("handle already freed")
        return self._h

    def info(self, what):
        return int(load_library().ubp_packed_info(self.handle, what))

    def layout(self, sub_stripes, col_tiles, which=1):
        """ubp_packed_layout, as copies.  which=1 (gather layout): (rg_ptr int32[nrg + 1], rg_order
        int32[nrg], stream uint32[...]); which=2 (block layout): (rg_ptr, rg_order int32[2 nrg + 1] = the
        order followed by the first stripe of every row group, records
        uint32[steps + spare][256], meta uint32[steps + spare][2]); which=3 (dense operand tiles):
        (None, None, uint16[stripes][tiles][64][8], occupied uint32[stripes][words])."""
        nrg = ctypes.c_int32(0)
        words, mwords = ctypes.c_int64(0), ctypes.c_int64(0)
        a, b, c, m = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        rc = load_library().ubp_packed_layout(self.handle, sub_stripes, col_tiles, which, ctypes.byref(nrg),
                                              ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(words),
                                              ctypes.byref(m), ctypes.byref(mwords))
        if rc != UBP_OK:
            raise UBPError(rc, "ubp_packed_layout")

        def copy(ptr, n, dt):
            if n == 0:
                return np.zeros(0, dtype=dt)
            buf = (ctypes.c_char * (n * np.dtype(dt).itemsize)).from_address(ptr.value)
            return np.frombuffer(buf, dtype=dt).copy()
        if which == 3:
            t = copy(c, words.value, np.uint32).view(np.uint16)
            return None, None, t.reshape(nrg.value, -1, 64, 8), copy(m, mwords.value, np.uint32).reshape(nrg.value, -1)
        rg_ptr = copy(a, nrg.value + 1, np.int32)
        rg_order = copy(b, nrg.value if which != 2 else 2 * nrg.value + 1, np.int32)
        if which == 2:
            return rg_ptr, rg_order, copy(c, words.value, np.uint32).reshape(-1, 256), copy(m, mwords.value, np.uint32).reshape(-1, 2)
        return rg_ptr, rg_order, copy(c, words.value, np.uint32)

    def _view(self, fn, np_dtype):
        n = ctypes.c_int64(0)
        ptr = fn(self.handle, ctypes.byref(n))
        if n.value == 0:
            return np.zeros(0, dtype=np_dtype)
        buf = (ctypes.c_char * (n.value * np.dtype(np_dtype).itemsize)).from_address(ptr)
        return np.frombuffer(buf, dtype=np_dtype).copy()

    @property
    def indptr(self):
        return self._view(load_library().ubp_packed_indptr, np.int32)

    @property
    def indices(self):
        return self._view(load_library().ubp_packed_indices, np.int32)

    @property
    def values(self):
        return self._view(load_library().ubp_packed_values, _NP_OF[self.dtype])

    def device_error(self):
        """Flags raised by a kernel whose bounded wait ran out (0 = healthy)."""
        flags = ctypes.c_uint32(0)
        rc = load_library().ubp_packed_device_error(self.handle, ctypes.byref(flags))
        if rc != UBP_OK:
            raise UBPError(rc, "ubp_packed_device_error")
        return int(flags.value)

    def free(self):
        if self._h:
            load_library().ubp_packed_free(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def pack(W_host, dtype, bh, bw, blocks, device=UBP_HOST_ONLY):
    """ubp_pack.  W_host: 2-D numpy array holding the element type's bits (float32, float16,
    or uint16 for bf16), row-major; blocks: [nb, 2] (r, c).  device: HIP ordinal or -1."""
    L = load_library()
    W = np.asarray(W_host)
    if W.ndim != 2 or W.dtype != _NP_OF[dtype] or W.strides[1] != W.itemsize or W.strides[0] % W.itemsize:
        raise ValueError("W must be a row-major 2-D array of %s" % _NP_OF[dtype].__name__)
    b = np.ascontiguousarray(np.asarray(blocks, dtype=np.int32).reshape(-1, 2))
    out = ctypes.c_void_p(None)
    rc = L.ubp_pack(W.ctypes.data, DTYPES[dtype], W.shape[0], W.shape[1], W.strides[0] // W.itemsize,
                    bh, bw, b.ctypes.data, b.shape[0], int(device), ctypes.byref(out))
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_pack")
    return Packed(out.value, dtype)


def spmm(packed, X_ptr, ldx, N, Y_ptr, ldy, y_dtype, stream=0, plan=None):
    """ubp_spmm / ubp_spmm_plan with raw DEVICE pointers (e.g. torch tensors' data_ptr())."""
    L = load_library()
    if plan is None:
        rc = L.ubp_spmm(packed.handle, X_ptr, ldx, N, Y_ptr, ldy, DTYPES[y_dtype], stream)
    else:
        rc = L.ubp_spmm_plan(packed.handle, X_ptr, ldx, N, Y_ptr, ldy, DTYPES[y_dtype], stream, ctypes.byref(plan))
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_spmm")


def spmm_fused(packed, X_ptr, ldx, N, Y_ptr, ldy, y_dtype, bias_ptr=None, activation=None, lo=0.0, hi=0.0, stream=0,
               plan=None):
    """ubp_spmm_fused with raw DEVICE pointers; bias_ptr: M floats on the device or None;
    activation: None / "relu" / "clamp" (with lo, hi)."""
    ep = Epilogue(bias_ptr, ACTIVATIONS[activation], float(lo), float(hi))
    rc = load_library().ubp_spmm_fused(packed.handle, X_ptr, ldx, N, Y_ptr, ldy, DTYPES[y_dtype], ctypes.byref(ep), stream,
                                       ctypes.byref(plan) if plan is not None else None)
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_spmm_fused")


def spmm_prepare(packed, X_ptr, ldx, N, Y_ptr, ldy, y_dtype, plan=None):
    """ubp_spmm_prepare: everything ubp_spmm / ubp_spmm_plan would do with these arguments except
    the launch.  Returns the resolved Plan."""
    chosen = Plan()
    rc = load_library().ubp_spmm_prepare(packed.handle, X_ptr, ldx, N, Y_ptr, ldy, DTYPES[y_dtype],
                                         ctypes.byref(plan) if plan is not None else None, ctypes.byref(chosen))
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_spmm_prepare")
    return chosen


def launch_floor(stream=0):
    """ubp_launch_floor: an empty kernel on the stream."""
    rc = load_library().ubp_launch_floor(stream)
    if rc != UBP_OK:
        raise UBPError(rc, "ubp_launch_floor")
