"""Thin ctypes binding over libe2f.so: argument marshalling only.

Function names follow include/e2f.h.  PyTorch supplies device memory and the current HIP stream; every step of
the operator runs inside the library's kernels.  Loading fails loudly when the library has not been built
(`python -m paper_2601_16622_amd.build`): there is no fallback path.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libe2f.so")

E2F_OK = 0
E2F_F32, E2F_BF16 = 0, 1
ATTENTION = {"auto": 0, "tile": 1, "pair": 2, "valu": 3}   # e2f_attn_kernel
E2F_FLAG_TILE_LISTS_PER_HEAD, E2F_FLAG_PROJECT_PER_CHANNEL_TILE = 1, 2

EXPORTS = ["e2f_status_string", "e2f_create", "e2f_destroy", "e2f_cells_workspace_bytes", "e2f_build_cells",
           "e2f_cells_destroy", "e2f_count_neighbors", "e2f_list_neighbors", "e2f_attn_workspace_bytes",
           "e2f_attn_forward", "e2f_attn_forward_materialized", "e2f_profile_begin", "e2f_profile_end",
           "e2f_eaas_tensor_product", "e2f_attn_factorized_workspace_bytes", "e2f_attn_forward_factorized",
           "e2f_attn_capped_workspace_bytes", "e2f_attn_forward_capped", "e2f_build_neighbor_table",
           "e2f_attn_table_workspace_bytes", "e2f_attn_forward_table", "e2f_build_cells_periodic",
           "e2f_attn_backward_workspace_bytes", "e2f_attn_backward", "e2f_attn_backward_after_forward",
           "e2f_attn_backward_weights_workspace_bytes", "e2f_attn_nonlinear_workspace_bytes",
           "e2f_attn_forward_nonlinear", "e2f_count_edges", "e2f_profile_read",
           "e2f_attn_forward_static"]
STATIC_SCRATCH_BYTES = 32 << 20   # E2F_STATIC_SCRATCH_BYTES
STAGES = ("prepare", "project", "attention")


class Config(ctypes.Structure):
    _fields_ = [("L_max", ctypes.c_int32), ("C", ctypes.c_int32), ("H", ctypes.c_int32), ("B", ctypes.c_int32),
                ("lf", ctypes.c_int32), ("cutoff", ctypes.c_float), ("feat_dtype", ctypes.c_int32),
                ("attention", ctypes.c_int32), ("flags", ctypes.c_int32)]


class Weights(ctypes.Structure):
    _fields_ = [(k, ctypes.c_void_p) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV", "Wb", "w_path")]


class E2fError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


_lib = None


def load():
    """Load libe2f.so and declare the signatures of include/e2f.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing - build it with `python -m paper_2601_16622_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    L.e2f_status_string.argtypes = [ctypes.c_int]
    L.e2f_status_string.restype = ctypes.c_char_p
    L.e2f_create.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(vp)]
    L.e2f_create.restype = ctypes.c_int
    L.e2f_destroy.argtypes = [vp]
    L.e2f_destroy.restype = None
    L.e2f_cells_workspace_bytes.argtypes = [vp, i32, i32]
    L.e2f_cells_workspace_bytes.restype = sz
    L.e2f_build_cells.argtypes = [vp, vp, vp, i32, i32, vp, sz, ctypes.POINTER(vp), vp]
    L.e2f_build_cells.restype = ctypes.c_int
    L.e2f_build_cells_periodic.argtypes = [vp, vp, vp, i32, i32, vp, vp, sz, ctypes.POINTER(vp), vp]
    L.e2f_build_cells_periodic.restype = ctypes.c_int
    L.e2f_cells_destroy.argtypes = [vp]
    L.e2f_cells_destroy.restype = None
    L.e2f_count_neighbors.argtypes = [vp, vp, vp, i32, vp, vp]
    L.e2f_count_neighbors.restype = ctypes.c_int
    L.e2f_list_neighbors.argtypes = [vp, vp, vp, i32, vp, vp, vp]
    L.e2f_list_neighbors.restype = ctypes.c_int
    L.e2f_count_edges.argtypes = [vp, vp, vp, i32, ctypes.POINTER(ctypes.c_int64), vp, vp]
    L.e2f_count_edges.restype = ctypes.c_int
    L.e2f_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32)]
    L.e2f_profile_read.restype = ctypes.c_int
    L.e2f_attn_workspace_bytes.argtypes = [vp, i32]
    L.e2f_attn_workspace_bytes.restype = sz
    L.e2f_attn_forward.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), vp, vp, sz, vp]
    L.e2f_attn_forward.restype = ctypes.c_int
    L.e2f_attn_forward_static.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), vp, vp]
    L.e2f_attn_forward_static.restype = ctypes.c_int
    L.e2f_attn_forward_materialized.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), vp, vp, sz, vp,
                                                ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.e2f_attn_forward_materialized.restype = ctypes.c_int
    L.e2f_attn_factorized_workspace_bytes.argtypes = [vp, i32]
    L.e2f_attn_factorized_workspace_bytes.restype = sz
    L.e2f_attn_forward_factorized.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), vp, vp, sz, vp]
    L.e2f_attn_forward_factorized.restype = ctypes.c_int
    L.e2f_attn_nonlinear_workspace_bytes.argtypes = [vp, i32]
    L.e2f_attn_nonlinear_workspace_bytes.restype = sz
    L.e2f_attn_forward_nonlinear.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), vp, vp, sz, vp]
    L.e2f_attn_forward_nonlinear.restype = ctypes.c_int
    L.e2f_attn_capped_workspace_bytes.argtypes = [vp, i32]
    L.e2f_attn_capped_workspace_bytes.restype = sz
    L.e2f_attn_forward_capped.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), i32, vp, vp, sz, vp]
    L.e2f_attn_forward_capped.restype = ctypes.c_int
    L.e2f_build_neighbor_table.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
    L.e2f_build_neighbor_table.restype = ctypes.c_int
    L.e2f_attn_table_workspace_bytes.argtypes = [vp, i32]
    L.e2f_attn_table_workspace_bytes.restype = sz
    L.e2f_attn_forward_table.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), vp, i32, vp, vp, sz, vp]
    L.e2f_attn_forward_table.restype = ctypes.c_int
    L.e2f_attn_backward_workspace_bytes.argtypes = [vp, i32]
    L.e2f_attn_backward_workspace_bytes.restype = sz
    L.e2f_attn_backward_weights_workspace_bytes.argtypes = [vp, i32]
    L.e2f_attn_backward_weights_workspace_bytes.restype = sz
    L.e2f_attn_backward.argtypes = [vp, vp, vp, vp, vp, i32, i32, ctypes.POINTER(Weights), vp, vp, vp, vp, vp, vp, vp,
                                    vp, vp, vp, vp, sz, vp]
    L.e2f_attn_backward.restype = ctypes.c_int
    L.e2f_attn_backward_after_forward.argtypes = L.e2f_attn_backward.argtypes
    L.e2f_attn_backward_after_forward.restype = ctypes.c_int
    L.e2f_eaas_tensor_product.argtypes = [vp, vp, vp, vp, vp, i32, vp]
    L.e2f_eaas_tensor_product.restype = ctypes.c_int
    L.e2f_profile_begin.argtypes = [vp, i32]
    L.e2f_profile_begin.restype = ctypes.c_int
    L.e2f_profile_end.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    L.e2f_profile_end.restype = ctypes.c_int
    _lib = L
    return L


def status_string(code):
    return load().e2f_status_string(int(code)).decode()


def _check(code, where):
    if code != E2F_OK:
        raise E2fError(code, where)


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None and t.numel() > 0 else 0)


def e2f_create(L_max, C, H, B, lf, cutoff, feat_dtype, attention="auto", flags=0):
    cfg = Config(L_max, C, H, B, lf, float(cutoff), E2F_BF16 if feat_dtype in ("bf16", E2F_BF16) else E2F_F32,
                 ATTENTION.get(attention, attention), int(flags))
    ctx = ctypes.c_void_p()
    _check(load().e2f_create(ctypes.byref(cfg), ctypes.byref(ctx)), "e2f_create")
    return ctx


def e2f_destroy(ctx):
    load().e2f_destroy(ctx)


def e2f_cells_workspace_bytes(ctx, N, S):
    return load().e2f_cells_workspace_bytes(ctx, N, S)


def e2f_build_cells(ctx, pos, seg_offsets, ws):
    """pos float32 [N][3], seg_offsets int32 [S+1], ws uint8 workspace (all CUDA tensors).  Returns the cells handle."""
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    cells = ctypes.c_void_p()
    _check(load().e2f_build_cells(ctx, _ptr(pos), _ptr(seg_offsets), N, S, _ptr(ws), ws.numel(), ctypes.byref(cells),
                                  _stream()), "e2f_build_cells")
    return cells


def e2f_build_cells_periodic(ctx, pos, seg_offsets, box, ws):
    """As e2f_build_cells, with box a host float32 array [S][3] of periodic edge lengths (<= 0: open axis) or None."""
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    cells = ctypes.c_void_p()
    if box is not None:
        box = np.ascontiguousarray(box, dtype=np.float32)
        assert box.shape == (S, 3)
    bptr = ctypes.c_void_p(box.ctypes.data) if box is not None else ctypes.c_void_p()
    _check(load().e2f_build_cells_periodic(ctx, _ptr(pos), _ptr(seg_offsets), N, S, bptr, _ptr(ws), ws.numel(),
                                           ctypes.byref(cells), _stream()), "e2f_build_cells_periodic")
    return cells


def e2f_cells_destroy(cells):
    load().e2f_cells_destroy(cells)


def e2f_count_neighbors(ctx, cells, pos, degree):
    _check(load().e2f_count_neighbors(ctx, cells, _ptr(pos), pos.shape[0], _ptr(degree), _stream()),
           "e2f_count_neighbors")


def e2f_count_edges(ctx, cells, pos, degree):
    """Returns E; degree (device int32 [N]) receives the neighbour counts."""
    E = ctypes.c_int64(0)
    _check(load().e2f_count_edges(ctx, cells, _ptr(pos), pos.shape[0], ctypes.byref(E), _ptr(degree), _stream()),
           "e2f_count_edges")
    return E.value


def e2f_list_neighbors(ctx, cells, pos, offsets, idx):
    _check(load().e2f_list_neighbors(ctx, cells, _ptr(pos), pos.shape[0], _ptr(offsets), _ptr(idx), _stream()),
           "e2f_list_neighbors")


def e2f_attn_workspace_bytes(ctx, N):
    return load().e2f_attn_workspace_bytes(ctx, N)


def _weights(w):
    return Weights(*[w[k].data_ptr() for k in ("WQ1", "WQ2", "WK1", "WK2", "WV", "Wb", "w_path")])


def e2f_attn_forward(ctx, cells, pos, h, seg_offsets, weights, out, ws):
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    wt = _weights(weights)
    _check(load().e2f_attn_forward(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S, ctypes.byref(wt),
                                   _ptr(out), _ptr(ws), ws.numel(), _stream()), "e2f_attn_forward")


def e2f_attn_forward_static(ctx, cells, pos, h, seg_offsets, weights, out):
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    wt = _weights(weights)
    _check(load().e2f_attn_forward_static(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S, ctypes.byref(wt),
                                          _ptr(out), _stream()), "e2f_attn_forward_static")


def e2f_attn_capped_workspace_bytes(ctx, N):
    return load().e2f_attn_capped_workspace_bytes(ctx, N)


def e2f_attn_forward_capped(ctx, cells, pos, h, seg_offsets, weights, max_neighbors, out, ws):
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    wt = _weights(weights)
    _check(load().e2f_attn_forward_capped(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S, ctypes.byref(wt),
                                          int(max_neighbors), _ptr(out), _ptr(ws), ws.numel(), _stream()),
           "e2f_attn_forward_capped")


def e2f_build_neighbor_table(ctx, cells, pos, K, table, count=None):
    _check(load().e2f_build_neighbor_table(ctx, cells, _ptr(pos), pos.shape[0], int(K), _ptr(table),
                                           _ptr(count) if count is not None else None, _stream()),
           "e2f_build_neighbor_table")


def e2f_attn_table_workspace_bytes(ctx, N):
    return load().e2f_attn_table_workspace_bytes(ctx, N)


def e2f_attn_forward_table(ctx, cells, pos, h, seg_offsets, weights, table, K, out, ws):
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    wt = _weights(weights)
    _check(load().e2f_attn_forward_table(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S, ctypes.byref(wt),
                                         _ptr(table), int(K), _ptr(out), _ptr(ws), ws.numel(), _stream()),
           "e2f_attn_forward_table")


def e2f_attn_nonlinear_workspace_bytes(ctx, N):
    return load().e2f_attn_nonlinear_workspace_bytes(ctx, N)


def e2f_attn_forward_nonlinear(ctx, cells, pos, h, seg_offsets, weights, out, ws):
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    wt = _weights(weights)
    _check(load().e2f_attn_forward_nonlinear(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S, ctypes.byref(wt),
                                             _ptr(out), _ptr(ws), ws.numel(), _stream()), "e2f_attn_forward_nonlinear")


def e2f_attn_factorized_workspace_bytes(ctx, N):
    return load().e2f_attn_factorized_workspace_bytes(ctx, N)


def e2f_attn_forward_factorized(ctx, cells, pos, h, seg_offsets, weights, out, ws):
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    wt = _weights(weights)
    _check(load().e2f_attn_forward_factorized(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S, ctypes.byref(wt),
                                              _ptr(out), _ptr(ws), ws.numel(), _stream()), "e2f_attn_forward_factorized")


def e2f_attn_backward_workspace_bytes(ctx, N):
    return load().e2f_attn_backward_workspace_bytes(ctx, N)


def e2f_attn_backward_weights_workspace_bytes(ctx, N):
    return load().e2f_attn_backward_weights_workspace_bytes(ctx, N)


def e2f_attn_backward_after_forward(ctx, cells, pos, h, seg_offsets, weights, out, grad_out, grad_pos, grad_q, grad_k,
                                    grad_v, grad_h, ws, grad_Wb=None, grad_w_path=None, grad_W=None):
    """ws: the workspace that the last e2f_attn_forward call for the same arguments wrote (see include/e2f.h)."""
    return e2f_attn_backward(ctx, cells, pos, h, seg_offsets, weights, out, grad_out, grad_pos, grad_q, grad_k, grad_v,
                             grad_h, ws, grad_Wb, grad_w_path, grad_W, entry="e2f_attn_backward_after_forward")


def e2f_attn_backward(ctx, cells, pos, h, seg_offsets, weights, out, grad_out, grad_pos, grad_q, grad_k, grad_v, grad_h,
                      ws, grad_Wb=None, grad_w_path=None, grad_W=None, entry="e2f_attn_backward"):
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    w = _weights(weights)
    _check(getattr(load(), entry)(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S, ctypes.byref(w), _ptr(out),
                                    _ptr(grad_out), _ptr(grad_pos), _ptr(grad_q), _ptr(grad_k), _ptr(grad_v),
                                    _ptr(grad_h) if grad_h is not None else ctypes.c_void_p(),
                                    _ptr(grad_Wb) if grad_Wb is not None else ctypes.c_void_p(),
                                    _ptr(grad_w_path) if grad_w_path is not None else ctypes.c_void_p(),
                                    _ptr(grad_W) if grad_W is not None else ctypes.c_void_p(),
                                    _ptr(ws), ws.numel(), _stream()), entry)


def e2f_attn_forward_materialized(ctx, cells, pos, h, seg_offsets, weights, out, ws):
    """Returns (n_edges, peak_bytes_allocated_inside)."""
    N, S = pos.shape[0], seg_offsets.shape[0] - 1
    wt = _weights(weights)
    edges, peak = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load().e2f_attn_forward_materialized(ctx, cells, _ptr(pos), _ptr(h), _ptr(seg_offsets), N, S,
                                                ctypes.byref(wt), _ptr(out), _ptr(ws), ws.numel(), _stream(),
                                                ctypes.byref(edges), ctypes.byref(peak)),
           "e2f_attn_forward_materialized")
    return edges.value, peak.value


def e2f_eaas_tensor_product(ctx, h, r, w_path, out):
    """h [T][n][C] (feature dtype), r float32 [T][3], w_path float32 [L+1][L+1], out float32 [T][n][C]."""
    _check(load().e2f_eaas_tensor_product(ctx, _ptr(h), _ptr(r), _ptr(w_path), _ptr(out), h.shape[0], _stream()),
           "e2f_eaas_tensor_product")


def e2f_profile_begin(ctx, max_calls):
    _check(load().e2f_profile_begin(ctx, max_calls), "e2f_profile_begin")


def e2f_profile_read(ctx, capacity):
    """Per-call stage times so far: list of {stage: ms}."""
    buf = (ctypes.c_float * (capacity * len(STAGES)))()
    calls = ctypes.c_int32(0)
    _check(load().e2f_profile_read(ctx, buf, capacity, ctypes.byref(calls)), "e2f_profile_read")
    return [{k: float(buf[c * len(STAGES) + i]) for i, k in enumerate(STAGES)} for c in range(calls.value)]


def e2f_profile_end(ctx):
    """Returns ({stage: mean ms}, calls)."""
    ms = (ctypes.c_float * len(STAGES))()
    calls = ctypes.c_int32(0)
    _check(load().e2f_profile_end(ctx, ms, ctypes.byref(calls)), "e2f_profile_end")
    return {k: float(ms[i]) for i, k in enumerate(STAGES)}, calls.value


class Problem:
    """Device-resident copy of one workload (see workloads.py) plus the library objects needed to run it."""

    def __init__(self, wl, device="cuda:0", attention="auto", flags=0):
        import torch
        cfg = wl["cfg"]
        self.cfg = cfg
        self.device = torch.device(device)
        fdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        self.N = wl["pos"].shape[0]
        self.S = wl["seg"].shape[0] - 1
        self.n = (cfg["L"] + 1) ** 2
        self.pos = torch.from_numpy(np.ascontiguousarray(wl["pos"], dtype=np.float32)).to(self.device)
        self.seg = torch.from_numpy(np.ascontiguousarray(wl["seg"], dtype=np.int32)).to(self.device)
        self.h = torch.from_numpy(np.ascontiguousarray(wl["h"], dtype=np.float32)).to(self.device).to(fdt).contiguous()
        self.weights = {}
        for k, v in wl["weights"].items():
            t = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(self.device)
            self.weights[k] = (t.to(fdt) if k.startswith("W") and k != "Wb" else t).contiguous()
        self.ctx = e2f_create(cfg["L"], cfg["C"], cfg["H"], cfg["B"], cfg["lf"], cfg["cutoff"], cfg["dtype"],
                              attention, flags)
        self.cells_ws = torch.empty(max(e2f_cells_workspace_bytes(self.ctx, self.N, self.S), 256), dtype=torch.uint8,
                                    device=self.device)
        self.attn_ws = torch.empty(max(e2f_attn_workspace_bytes(self.ctx, self.N), 256), dtype=torch.uint8,
                                   device=self.device)
        self.out = torch.empty((self.N, self.n, cfg["C"]), dtype=torch.float32, device=self.device)
        self.cells = None
        self.box = wl.get("box")   # host float32 [S][3] of periodic edge lengths, or None

    def build_cells(self):
        if self.cells is not None:
            e2f_cells_destroy(self.cells)
            self.cells = None
        if self.box is not None:
            self.cells = e2f_build_cells_periodic(self.ctx, self.pos, self.seg, self.box, self.cells_ws)
        else:
            self.cells = e2f_build_cells(self.ctx, self.pos, self.seg, self.cells_ws)
        return self.cells

    def forward(self, for_backward=False):
        """for_backward: run in the backward pass's workspace, so that backward(after_forward=True) can follow."""
        ws = self.attn_ws
        if for_backward:
            ws = self._scratch("bwd_ws", e2f_attn_backward_weights_workspace_bytes(self.ctx, self.N))
        e2f_attn_forward(self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, self.out, ws)
        return self.out

    def forward_static(self, out=None):
        out = self.out if out is None else out
        e2f_attn_forward_static(self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, out)
        return out

    def _scratch(self, name, need):
        import torch
        buf = getattr(self, name, None)
        if buf is None or buf.numel() < need:
            buf = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
            setattr(self, name, buf)
        return buf

    def forward_capped(self, max_neighbors, out=None):
        out = self.out if out is None else out
        ws = self._scratch("cap_ws", e2f_attn_capped_workspace_bytes(self.ctx, self.N))
        e2f_attn_forward_capped(self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, max_neighbors, out, ws)
        return out

    def neighbor_table(self, K):
        """(table [N][K] int32, count [N] int32) on the device."""
        import torch
        table = torch.empty((max(self.N, 1), K), dtype=torch.int32, device=self.device)
        count = torch.empty((max(self.N, 1),), dtype=torch.int32, device=self.device)
        e2f_build_neighbor_table(self.ctx, self.cells, self.pos, K, table, count)
        return table, count

    def forward_table(self, table, out=None):
        out = self.out if out is None else out
        ws = self._scratch("table_ws", e2f_attn_table_workspace_bytes(self.ctx, self.N))
        e2f_attn_forward_table(self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, table, table.shape[1], out, ws)
        return out

    def forward_nonlinear(self, out=None):
        out = self.out if out is None else out
        ws = self._scratch("nonlinear_ws", e2f_attn_nonlinear_workspace_bytes(self.ctx, self.N))
        e2f_attn_forward_nonlinear(self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, out, ws)
        return out

    def forward_factorized(self, out=None):
        import torch
        out = self.out if out is None else out
        need = e2f_attn_factorized_workspace_bytes(self.ctx, self.N)
        if getattr(self, "fact_ws", None) is None or self.fact_ws.numel() < need:
            self.fact_ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        e2f_attn_forward_factorized(self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, out, self.fact_ws)
        return out

    def backward(self, grad_out, out=None, with_h=True, with_weights=False, after_forward=False):
        """Gradients of sum(out * grad_out): (grad_pos [N][3], grad_q, grad_k [N][L+1][C], grad_v [N][n][C],
        grad_h [N][n][C] or None); with_weights appends (grad_Wb [H][B], grad_w_path [L+1][L+1],
        grad_W [5][L+1][C][C]).  after_forward: e2f_attn_backward_after_forward, right after forward(for_backward=True)."""
        import torch
        out = self.out if out is None else out
        need = (e2f_attn_backward_weights_workspace_bytes if with_weights else e2f_attn_backward_workspace_bytes)(self.ctx, self.N)
        ws = self._scratch("bwd_ws", need)
        L1 = self.cfg["L"] + 1
        gp = torch.empty((self.N, 3), dtype=torch.float32, device=self.device)
        gq = torch.empty((self.N, L1, self.cfg["C"]), dtype=torch.float32, device=self.device)
        gk = torch.empty_like(gq)
        gv = torch.empty((self.N, self.n, self.cfg["C"]), dtype=torch.float32, device=self.device)
        gh = torch.empty_like(gv) if with_h else None
        gwb = gwp = gw = None
        if with_weights:
            C = self.cfg["C"]
            gwb = torch.empty((self.cfg["H"], self.cfg["B"]), dtype=torch.float32, device=self.device)
            gwp = torch.empty((L1, L1), dtype=torch.float32, device=self.device)
            gw = torch.empty((5, L1, C, C), dtype=torch.float32, device=self.device)
        (e2f_attn_backward_after_forward if after_forward else e2f_attn_backward)(
            self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, out, grad_out, gp, gq, gk, gv, gh, ws, gwb, gwp, gw)
        return (gp, gq, gk, gv, gh, gwb, gwp, gw) if with_weights else (gp, gq, gk, gv, gh)

    def forward_materialized(self, out=None):
        out = self.out if out is None else out
        return e2f_attn_forward_materialized(self.ctx, self.cells, self.pos, self.h, self.seg, self.weights, out,
                                             self.attn_ws)

    def neighbors(self):
        """(degree int32 [N], offsets int64 [N+1], idx int32 [E]) as numpy arrays, rows sorted."""
        import torch
        deg = torch.zeros(self.N, dtype=torch.int32, device=self.device)
        e2f_count_neighbors(self.ctx, self.cells, self.pos, deg)
        offsets = torch.zeros(self.N + 1, dtype=torch.int64, device=self.device)
        offsets[1:] = torch.cumsum(deg.to(torch.int64), 0)
        E = int(offsets[-1].item())
        idx = torch.full((max(E, 1),), -1, dtype=torch.int32, device=self.device)
        e2f_list_neighbors(self.ctx, self.cells, self.pos, offsets, idx)
        torch.cuda.synchronize()
        offs = offsets.cpu().numpy()
        idx = idx.cpu().numpy()[:E]
        for i in range(self.N):
            idx[offs[i]:offs[i + 1]].sort()
        return deg.cpu().numpy(), offs, idx

    def activation_bytes(self):
        return self.attn_ws.numel() + self.out.numel() * 4

    def close(self):
        if self.cells is not None:
            e2f_cells_destroy(self.cells)
            self.cells = None
        if self.ctx is not None:
            e2f_destroy(self.ctx)
            self.ctx = None
