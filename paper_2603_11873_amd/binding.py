"""ctypes binding with the same names as the C ABI (include/adafuse.h)."""
import ctypes as C
import os

PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(PKG, "libadafuse.so")
_lib = None

MERGE, UNMERGE, SWAP = 0, 1, 2
GATE_SOFTMAX_OVER_TOPK, GATE_TOPK_OF_SOFTMAX = 0, 1
KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA, KERNEL_GEMM = 0, 1, 2, 3
OPT_KERNEL, OPT_GEMM_WAVES, OPT_GEMM_FORM, OPT_XCD_RUN, OPT_PANEL_KB, OPT_MFMA_SHAPE = range(6)
PROBE_READ_BASE, PROBE_ZERO_WORK = 0, 1

EXPORTS = ["adafuse_create", "adafuse_destroy", "adafuse_set_option", "adafuse_get_info",
           "adafuse_pregate", "adafuse_fused_switch", "adafuse_switch_per_matrix", "adafuse_forward_merged", "adafuse_forward_dynamic",
           "adafuse_forward_dynamic_static", "adafuse_prefill", "adafuse_prefill_workspace_bytes", "adafuse_prefill_group", "adafuse_prefill_group_workspace_bytes", "adafuse_hbm_probe", "adafuse_switch_kernel_name", "adafuse_status_string"]


class AdafuseError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        msg = load_library().adafuse_status_string(self.status).decode()
        super().__init__(f"{what}: {msg} (status {self.status})")


class MatrixDesc(C.Structure):
    """adafuse_matrix_desc"""
    _fields_ = [("w_base", C.c_void_p), ("w_work", C.c_void_p), ("a_bank", C.c_void_p), ("b_bank", C.c_void_p),
                ("out", C.c_int32), ("in_", C.c_int32), ("ldw", C.c_int32), ("reserved", C.c_int32)]


class Info(C.Structure):
    """adafuse_info"""
    _fields_ = [("n_mats", C.c_int32), ("E", C.c_int32), ("r", C.c_int32), ("k_max", C.c_int32),
                ("kernel", C.c_int32), ("tile_rows", C.c_int32), ("tile_cols", C.c_int32), ("reserved", C.c_int32),
                ("n_tiles", C.c_int64), ("elements", C.c_int64)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libadafuse.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2603_11873_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(_LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    L.adafuse_create.restype = i32
    L.adafuse_create.argtypes = [C.POINTER(MatrixDesc), i32, i32, i32, i32, C.POINTER(vp)]
    L.adafuse_destroy.restype = i32
    L.adafuse_destroy.argtypes = [vp]
    L.adafuse_set_option.restype = i32
    L.adafuse_set_option.argtypes = [vp, i32, i32]
    L.adafuse_get_info.restype = i32
    L.adafuse_get_info.argtypes = [vp, C.POINTER(Info)]
    L.adafuse_pregate.restype = i32
    L.adafuse_pregate.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    L.adafuse_fused_switch.restype = i32
    L.adafuse_fused_switch.argtypes = [vp, vp, vp, vp, vp, i32, f32, i32, vp]
    L.adafuse_switch_per_matrix.restype = i32
    L.adafuse_switch_per_matrix.argtypes = [vp, vp, vp, vp, vp, i32, f32, i32, vp]
    L.adafuse_forward_merged.restype = i32
    L.adafuse_forward_merged.argtypes = [vp, vp, vp, vp]
    L.adafuse_forward_dynamic.restype = i32
    L.adafuse_forward_dynamic.argtypes = [vp, C.POINTER(i32), C.POINTER(f32), i32, f32, vp, vp, vp, vp]
    L.adafuse_forward_dynamic_static.restype = i32
    L.adafuse_forward_dynamic_static.argtypes = [vp, C.POINTER(i32), C.POINTER(f32), i32, f32, vp, vp, vp]
    L.adafuse_prefill.restype = i32
    L.adafuse_prefill.argtypes = [vp, i32, vp, i32, vp, vp, i32, f32, vp, vp, C.c_size_t, vp]
    L.adafuse_prefill_workspace_bytes.restype = i32
    L.adafuse_prefill_workspace_bytes.argtypes = [vp, i32, i32, i32, C.POINTER(C.c_size_t)]
    L.adafuse_prefill_group.restype = i32
    L.adafuse_prefill_group.argtypes = [vp, C.POINTER(i32), i32, vp, i32, vp, vp, i32, f32, C.POINTER(vp), vp, C.c_size_t, vp]
    L.adafuse_prefill_group_workspace_bytes.restype = i32
    L.adafuse_prefill_group_workspace_bytes.argtypes = [vp, C.POINTER(i32), i32, i32, i32, C.POINTER(C.c_size_t)]
    L.adafuse_hbm_probe.restype = i32
    L.adafuse_hbm_probe.argtypes = [vp, i32, vp]
    L.adafuse_switch_kernel_name.restype = C.c_char_p
    L.adafuse_switch_kernel_name.argtypes = [vp, i32, i32]
    L.adafuse_status_string.restype = C.c_char_p
    L.adafuse_status_string.argtypes = [i32]
    _lib = L
    return L


def _ptr(t):
    """Device (or host) address of a torch tensor, or NULL."""
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def pregate(hidden, w_router, k, gate_norm=GATE_SOFTMAX_OVER_TOPK, want_logits=True, stream=None, out=None):
    """adafuse_pregate on torch tensors: hidden bf16 [T][d], w_router bf16 [E][d] (device).

    Returns (idx int32 [T][k], gates fp32 [T][k], logits fp32 [T][E] or None), device tensors
    written asynchronously on `stream` (default: torch's current stream).
    """
    import torch
    T, d = hidden.shape
    E = w_router.shape[0]
    assert hidden.dtype == torch.bfloat16 and w_router.dtype == torch.bfloat16
    assert hidden.is_contiguous() and w_router.is_contiguous() and w_router.shape[1] == d
    if out is None:
        idx = torch.empty((T, k), dtype=torch.int32, device=hidden.device)
        gates = torch.empty((T, k), dtype=torch.float32, device=hidden.device)
        logits = torch.empty((T, E), dtype=torch.float32, device=hidden.device) if want_logits else None
    else:
        idx, gates, logits = out
    st = load_library().adafuse_pregate(_ptr(hidden), _ptr(w_router), T, d, E, k, gate_norm,
                                        _ptr(idx), _ptr(gates), _ptr(logits), _stream_handle(stream))
    if st != 0:
        raise AdafuseError(st, "adafuse_pregate")
    return idx, gates, logits


class Context:
    """adafuse_ctx: a fixed set of adapted matrices.

    mats: list of (w_base, w_work, a_bank, b_bank) torch bf16 device tensors with
    shapes [out][in], [out][in], [E][r][in], [E][out][r].  The context keeps
    references so the memory outlives it.
    """

    def __init__(self, mats, k_max):
        import torch
        self._keep = list(mats)
        n = len(self._keep)
        arr = (MatrixDesc * max(n, 1))()
        E = r = None
        for i, (wb, ww, a, b) in enumerate(self._keep):
            for t in (wb, ww, a, b):
                assert t.dtype == torch.bfloat16 and t.is_cuda
            assert a.is_contiguous() and b.is_contiguous()
            out, in_ = wb.shape
            assert ww.shape == wb.shape and wb.stride(1) == 1 and ww.stride(1) == 1 and wb.stride(0) == ww.stride(0)
            assert a.shape[0] == b.shape[0] and a.shape[2] == in_ and b.shape[1] == out and a.shape[1] == b.shape[2]
            if E is None:
                E, r = a.shape[0], a.shape[1]
            assert (E, r) == (a.shape[0], a.shape[1])
            arr[i] = MatrixDesc(wb.data_ptr(), ww.data_ptr(), a.data_ptr(), b.data_ptr(), out, in_, wb.stride(0), 0)
        self.E, self.r, self.k_max = E or 0, r or 0, k_max
        self._h = C.c_void_p()
        st = load_library().adafuse_create(arr, n, self.E, self.r, k_max, C.byref(self._h))
        if st != 0:
            raise AdafuseError(st, "adafuse_create")

    def set_option(self, option, value):
        """adafuse_set_option"""
        st = load_library().adafuse_set_option(self._h, option, value)
        if st != 0:
            raise AdafuseError(st, "adafuse_set_option")

    def set_kernel(self, kernel):
        """adafuse_set_option(ADAFUSE_OPT_KERNEL, kernel)"""
        self.set_option(OPT_KERNEL, kernel)

    def info(self) -> Info:
        info = Info()
        st = load_library().adafuse_get_info(self._h, C.byref(info))
        if st != 0:
            raise AdafuseError(st, "adafuse_get_info")
        return info

    def switch_kernel_name(self, k, mode):
        """adafuse_switch_kernel_name: the device function a switch with these arguments launches, or None."""
        name = load_library().adafuse_switch_kernel_name(self._h, k, mode)
        return None if name is None else name.decode()

    def hbm_probe(self, direction, stream=None):
        """adafuse_hbm_probe: PROBE_READ_BASE reads every w_base tile, PROBE_ZERO_WORK zeroes every w_work tile."""
        st = load_library().adafuse_hbm_probe(self._h, direction, _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_hbm_probe")

    def fused_switch(self, idx_prev, gates_prev, idx_next, gates_next, k, scale, mode, stream=None):
        """adafuse_fused_switch; idx/gates are device tensors (int32[k] / fp32[k]) or None."""
        st = load_library().adafuse_fused_switch(self._h, _ptr(idx_prev), _ptr(gates_prev), _ptr(idx_next),
                                                 _ptr(gates_next), k, scale, mode, _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_fused_switch")

    def switch_per_matrix(self, idx_prev, gates_prev, idx_next, gates_next, k, scale, mode, stream=None):
        """adafuse_switch_per_matrix: same update, one launch per matrix (the paper's "simple merge")."""
        st = load_library().adafuse_switch_per_matrix(self._h, _ptr(idx_prev), _ptr(gates_prev), _ptr(idx_next),
                                                      _ptr(gates_next), k, scale, mode, _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_switch_per_matrix")

    def forward_merged(self, x, y, stream=None):
        """adafuse_forward_merged: y_m = W_work,m x_m for every matrix (x bf16, y fp32, concatenated)."""
        st = load_library().adafuse_forward_merged(self._h, _ptr(x), _ptr(y), _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_forward_merged")

    def forward_dynamic(self, idx, gates, scale, x, y, z, stream=None):
        """adafuse_forward_dynamic: the un-merged adapter path; idx/gates are host sequences."""
        k = len(idx)
        ci = (C.c_int32 * k)(*[int(v) for v in idx])
        cg = (C.c_float * k)(*[float(v) for v in gates])
        st = load_library().adafuse_forward_dynamic(self._h, ci, cg, k, scale, _ptr(x), _ptr(y), _ptr(z),
                                                    _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_forward_dynamic")

    def forward_dynamic_static(self, idx, gates, scale, x, y, stream=None):
        """adafuse_forward_dynamic_static: forward_dynamic with the library's built-in scratch (no workspace)."""
        k = len(idx)
        ci = (C.c_int32 * k)(*[int(v) for v in idx])
        cg = (C.c_float * k)(*[float(v) for v in gates])
        st = load_library().adafuse_forward_dynamic_static(self._h, ci, cg, k, scale, _ptr(x), _ptr(y),
                                                           _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_forward_dynamic_static")

    def prefill_workspace_bytes(self, mat, T, k):
        """adafuse_prefill_workspace_bytes"""
        n = C.c_size_t(0)
        st = load_library().adafuse_prefill_workspace_bytes(self._h, mat, T, k, C.byref(n))
        if st != 0:
            raise AdafuseError(st, "adafuse_prefill_workspace_bytes")
        return int(n.value)

    def prefill(self, mat, x, idx, gates, scale, y=None, workspace=None, stream=None):
        """adafuse_prefill: x bf16 [T][in], idx int32 [T][k], gates fp32 [T][k] (device) -> y fp32 [T][out]."""
        import torch
        T, k = idx.shape
        out = self._keep[mat][0].shape[0] if 0 <= mat < len(self._keep) else 0   # a bad index is the library's to refuse
        assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[0] == T
        assert idx.is_contiguous() and gates.is_contiguous() and gates.shape == idx.shape
        if y is None:
            y = torch.empty((T, out), dtype=torch.float32, device=x.device)
        if workspace is None:
            workspace = torch.empty(max(16, self.prefill_workspace_bytes(mat, T, k)), dtype=torch.uint8, device=x.device)
        st = load_library().adafuse_prefill(self._h, mat, _ptr(x), T, _ptr(idx), _ptr(gates), k, scale, _ptr(y),
                                            _ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_prefill")
        return y

    def prefill_group_workspace_bytes(self, mats, T, k):
        """adafuse_prefill_group_workspace_bytes"""
        n = C.c_size_t(0)
        arr = (C.c_int32 * len(mats))(*mats)
        st = load_library().adafuse_prefill_group_workspace_bytes(self._h, arr, len(mats), T, k, C.byref(n))
        if st != 0:
            raise AdafuseError(st, "adafuse_prefill_group_workspace_bytes")
        return int(n.value)

    def prefill_group(self, mats, x, idx, gates, scale, ys=None, workspace=None, stream=None):
        """adafuse_prefill_group: the matrices `mats` (same input width) applied to x bf16 [T][in] with per-token
        decisions idx / gates (device) -> list of y fp32 [T][out_i]."""
        import torch
        T, k = idx.shape
        assert x.dtype == torch.bfloat16 and x.is_contiguous() and x.shape[0] == T
        assert idx.is_contiguous() and gates.is_contiguous() and gates.shape == idx.shape
        if ys is None:
            ys = [torch.empty((T, self._keep[m][0].shape[0] if 0 <= m < len(self._keep) else 0), dtype=torch.float32,
                              device=x.device) for m in mats]
        if workspace is None:
            workspace = torch.empty(max(16, self.prefill_group_workspace_bytes(mats, T, k)), dtype=torch.uint8, device=x.device)
        arr = (C.c_int32 * len(mats))(*mats)
        yp = (C.c_void_p * len(mats))(*[_ptr(y) for y in ys])
        st = load_library().adafuse_prefill_group(self._h, arr, len(mats), _ptr(x), T, _ptr(idx), _ptr(gates), k, scale, yp,
                                                  _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                  _stream_handle(stream))
        if st != 0:
            raise AdafuseError(st, "adafuse_prefill_group")
        return ys

    def close(self):
        if self._h:
            load_library().adafuse_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
