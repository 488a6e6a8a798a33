"""ctypes access to the fp64 CPU oracle (oracle/e2f_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg
of bench.py.  Nothing in the product package imports this module, and this module imports nothing
from the product package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "e2f_oracle.c")
_LIB = os.path.join(_HERE, "libe2f_oracle.so")


def build(force=False):
    """Compile the oracle with gcc (host only).  -ffp-contract=off keeps the binary32 cutoff predicate free of FMA."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Config(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int), ("C", ctypes.c_int), ("H", ctypes.c_int), ("B", ctypes.c_int),
                ("lf", ctypes.c_int), ("cutoff", ctypes.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lp = ctypes.POINTER(ctypes.c_int64)
        L.e2fo_solid_harmonics.argtypes = [ctypes.c_int, dp, dp]
        L.e2fo_solid_harmonics.restype = None
        L.e2fo_cg_complex.argtypes = [ctypes.c_int] * 6
        L.e2fo_cg_complex.restype = ctypes.c_double
        L.e2fo_cg_real.argtypes = [ctypes.c_int] * 3 + [dp]
        L.e2fo_cg_real.restype = None
        L.e2fo_wigner_D_real.argtypes = [ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double, dp]
        L.e2fo_wigner_D_real.restype = None
        L.e2fo_align_angles.argtypes = [dp, dp, dp]
        L.e2fo_align_angles.restype = None
        L.e2fo_P_path.argtypes = [ctypes.c_int] * 3 + [ip, dp]
        L.e2fo_P_path.restype = ctypes.c_int
        L.e2fo_message.argtypes = [ctypes.c_int, ctypes.c_int, dp, dp, ctypes.c_int, dp, ctypes.c_int,
                                   ctypes.c_double, dp]
        L.e2fo_message.restype = None
        L.e2fo_neighbor_list.argtypes = [dp, ip, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_int, lp,
                                         ctypes.POINTER(ip)]
        L.e2fo_neighbor_list.restype = ctypes.c_int
        L.e2fo_free.argtypes = [ctypes.c_void_p]
        L.e2fo_free.restype = None
        L.e2fo_attn_forward.argtypes = [ctypes.POINTER(_Config), dp, dp, ctypes.c_int, dp, dp, dp, dp, dp, dp, dp,
                                        lp, ip, dp, ip, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                        ctypes.c_int, dp]
        L.e2fo_attn_forward.restype = ctypes.c_int
        L.e2fo_num_threads.argtypes = []
        L.e2fo_num_threads.restype = ctypes.c_int
        L.e2fo_set_num_threads.argtypes = [ctypes.c_int]
        L.e2fo_set_num_threads.restype = None
        _lib = L
    return _lib


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads():
    return lib().e2fo_num_threads()


def set_num_threads(n):
    """Thread count of the oracle's loops over target atoms (timing aid only; results do not depend on it)."""
    lib().e2fo_set_num_threads(int(n))


def solid_harmonics(l, r):
    r = _f64(r)
    out = np.empty(2 * l + 1)
    lib().e2fo_solid_harmonics(l, _d(r), _d(out))
    return out


def cg_complex(j1, m1, j2, m2, j, m):
    return lib().e2fo_cg_complex(j1, m1, j2, m2, j, m)


def cg_real(li, lf, lo):
    """Real-basis CG tensor [2lo+1][2li+1][2lf+1]."""
    out = np.empty((2 * lo + 1, 2 * li + 1, 2 * lf + 1))
    lib().e2fo_cg_real(li, lf, lo, _d(out))
    return out


def wigner_D_real(l, alpha, beta, gamma):
    """Real-basis D(Rz(alpha) Ry(beta) Rz(gamma)) with Y(R x) = D Y(x)."""
    out = np.empty((2 * l + 1, 2 * l + 1))
    lib().e2fo_wigner_D_real(l, alpha, beta, gamma, _d(out))
    return out


def align_angles(r):
    r = _f64(r)
    th, ph = ctypes.c_double(), ctypes.c_double()
    lib().e2fo_align_angles(_d(r), ctypes.byref(th), ctypes.byref(ph))
    return th.value, ph.value


def P_path(li, lf, lo):
    """(src, coef, worst): for each mo the one contributing input offset (or -1), its coefficient, and the
    largest number of contributing inputs found for any mo."""
    src = np.empty(2 * lo + 1, dtype=np.int32)
    coef = np.empty(2 * lo + 1)
    worst = lib().e2fo_P_path(li, lf, lo, src.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _d(coef))
    return src, coef, worst


def message(L, lf, w_path, v, r, mode="dense", chi=0.0):
    """Edge message for one pair; v is [(L+1)^2] or [(L+1)^2][C]."""
    v = _f64(v)
    squeeze = v.ndim == 1
    v2 = np.ascontiguousarray(v.reshape(v.shape[0], -1))
    w = _f64(w_path)
    r = _f64(r)
    out = np.empty_like(v2)
    lib().e2fo_message(L, lf, _d(w), _d(v2), v2.shape[1], _d(r), 0 if mode == "dense" else 1, float(chi), _d(out))
    return out[:, 0] if squeeze else out


def neighbor_list(pos, seg_offsets, cutoff, use_cells=False):
    """CSR neighbour lists (offsets int64[N+1], idx int32[E]); neighbours sorted by index."""
    pos = _f64(pos)
    seg = np.ascontiguousarray(seg_offsets, dtype=np.int32)
    N, S = pos.shape[0], seg.shape[0] - 1
    offsets = np.empty(N + 1, dtype=np.int64)
    ptr = ctypes.POINTER(ctypes.c_int32)()
    lib().e2fo_neighbor_list(_d(pos),
                             seg.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), N, S, ctypes.c_float(cutoff),
                             1 if use_cells else 0, offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                             ctypes.byref(ptr))
    E = int(offsets[-1])
    idx = np.ctypeslib.as_array(ptr, shape=(max(E, 1),))[:E].copy()
    lib().e2fo_free(ptr)
    return offsets, idx


def wrap_positions(pos, seg_offsets, box):
    """Coordinates folded into the periodic box, in binary32 with every operation rounded:
    q = floor(x * inv), inv = 1/len rounded to binary32;  w = x - len*q;  w < 0: w += len;  w >= len: w -= len.
    box is float [S][3], the edge lengths of every segment's orthorhombic box; an entry <= 0 leaves that axis open.
    Periodic boundaries are not part of the paper's operator (it takes the pair vectors as given); this is the
    convention of this build, used for the bulk simulations of the paper's Sec. 4.3."""
    p = np.array(pos, dtype=np.float32)
    box = np.asarray(box, dtype=np.float32).reshape(-1, 3)
    seg = np.asarray(seg_offsets)
    for s in range(len(seg) - 1):
        a0, a1 = int(seg[s]), int(seg[s + 1])
        for k in range(3):
            ln = np.float32(box[s, k])
            if not ln > 0:
                continue
            inv = np.float32(1.0) / ln
            x = p[a0:a1, k]
            q = np.floor(x * inv)
            w = x - ln * q
            w = np.where(w < 0, w + ln, w)
            w = np.where(w >= ln, w - ln, w)
            assert w.dtype == np.float32
            p[a0:a1, k] = w
    return p


def neighbor_list_periodic(pos, seg_offsets, cutoff, box):
    """Neighbour sets under periodic boundaries by brute force over all pairs of a segment.  With w the folded
    coordinates (wrap_positions), the image of j seen from i along a periodic axis of length len is
    w_j + s*len with s = +1 if w_i - w_j > len/2, s = -1 if w_j - w_i > len/2, else 0 (binary32); the predicate is
    the binary32 one of the open case on the image position fl(w_j + s*len).  Every periodic edge length must be at
    least three cutoffs, so at most one image of an atom lies within the cutoff.
    Returns (offsets int64 [N+1], idx int32 [E] sorted within a row, shift int8 [E][3])."""
    w = wrap_positions(pos, seg_offsets, box)
    box = np.asarray(box, dtype=np.float32).reshape(-1, 3)
    seg = np.asarray(seg_offsets)
    N = w.shape[0]
    rc2 = np.float32(cutoff) * np.float32(cutoff)
    offsets = np.zeros(N + 1, dtype=np.int64)
    rows_idx, rows_shift = [], []
    for s in range(len(seg) - 1):
        a0, a1 = int(seg[s]), int(seg[s + 1])
        ws = w[a0:a1]
        for i in range(a0, a1):
            d = []
            sh = np.zeros((a1 - a0, 3), dtype=np.int8)
            for k in range(3):
                ln = np.float32(box[s, k])
                xj = ws[:, k]
                if ln > 0:
                    half = ln * np.float32(0.5)
                    sk = np.where(w[i, k] - xj > half, 1, np.where(xj - w[i, k] > half, -1, 0)).astype(np.int8)
                    sh[:, k] = sk
                    xj = xj + sk.astype(np.float32) * ln
                d.append(xj - w[i, k])
            d2 = (d[0] * d[0] + d[1] * d[1]) + d[2] * d[2]
            assert d2.dtype == np.float32
            ok = (d2 < rc2) & (d2 > 0)
            ok[i - a0] = False
            nb = np.nonzero(ok)[0]
            rows_idx.append((nb + a0).astype(np.int32))
            rows_shift.append(sh[nb])
            offsets[i + 1] = offsets[i] + len(nb)
    idx = np.concatenate(rows_idx) if rows_idx else np.zeros(0, dtype=np.int32)
    shift = np.concatenate(rows_shift) if rows_shift else np.zeros((0, 3), dtype=np.int8)
    return offsets, idx.astype(np.int32), shift.astype(np.int8)


def edge_translations(seg_offsets, box, offsets, shift):
    """Lattice translation of every edge's neighbour image, float64 [E][3]: shift * box of the edge's segment."""
    box = np.asarray(box, dtype=np.float32).reshape(-1, 3).astype(np.float64)
    seg = np.asarray(seg_offsets)
    N = len(offsets) - 1
    atom_seg = np.repeat(np.arange(len(seg) - 1), np.diff(seg))
    edge_atom = np.repeat(np.arange(N), np.diff(offsets))
    return shift.astype(np.float64) * np.maximum(box[atom_seg[edge_atom]], 0.0)


def attn_forward(cfg, pos, h, seg_offsets, weights, targets=None, message_mode="dense", softmax_mode="twopass",
                 use_cells=False, chi=0.0, nbr=None, box=None, score_mode="kernel_score"):
    """The operator.  cfg: dict(L, C, H, B, lf, cutoff); weights: dict(WQ1, WQ2, WK1, WK2, WV [L+1][C][C],
    Wb [H][B], w_path [L+1][L+1]); returns float64 [n_targets][(L+1)^2][C].
    box: None, or float [S][3] periodic edge lengths (see neighbor_list_periodic); nbr is then the triple that
    function returns, and the pair vectors are r_ij = (w_j + shift*box) - w_i on the folded coordinates w.
    score_mode: "kernel_score" (Eq. kernel_score) or "nonlinear" (the logit with the non-linear pair feature of
    Eqs. app-nonlin-fea / app-nonlin-alpha, in the reading stated at e2fo_attn_forward)."""
    if score_mode not in ("kernel_score", "nonlinear"):
        raise ValueError("unknown score_mode")
    c = _Config(cfg["L"], cfg["C"], cfg["H"], cfg["B"], cfg["lf"], float(np.float32(cfg["cutoff"])))
    edge_shift = None
    if box is not None:
        if nbr is None:
            nbr = neighbor_list_periodic(pos, seg_offsets, np.float32(cfg["cutoff"]), box)
        edge_shift = np.ascontiguousarray(edge_translations(seg_offsets, box, nbr[0], nbr[2]))
        if edge_shift.size == 0:
            edge_shift = np.zeros((1, 3))
        pos = wrap_positions(pos, seg_offsets, box)
        nbr = (nbr[0], nbr[1])
    pos = _f64(pos)
    h = _f64(h)
    N = pos.shape[0]
    n = (cfg["L"] + 1) ** 2
    assert h.shape == (N, n, cfg["C"])
    if nbr is None:
        nbr = neighbor_list(pos, seg_offsets, np.float32(cfg["cutoff"]), use_cells)
    offsets, idx = nbr
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.size == 0:
        idx = np.zeros(1, dtype=np.int32)
    W = {k: _f64(weights[k]) for k in ("WQ1", "WQ2", "WK1", "WK2", "WV", "Wb", "w_path")}
    ip = ctypes.POINTER(ctypes.c_int32)
    if targets is None:
        tptr, nt = ip(), N
    else:
        targets = np.ascontiguousarray(targets, dtype=np.int32)
        tptr, nt = targets.ctypes.data_as(ip), targets.shape[0]
    out = np.empty((nt, n, cfg["C"]))
    rc = lib().e2fo_attn_forward(ctypes.byref(c), _d(pos), _d(h), N,
                                 _d(W["WQ1"]), _d(W["WQ2"]), _d(W["WK1"]), _d(W["WK2"]), _d(W["WV"]), _d(W["Wb"]),
                                 _d(W["w_path"]), offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                 idx.ctypes.data_as(ip),
                                 _d(edge_shift) if edge_shift is not None else ctypes.POINTER(ctypes.c_double)(),
                                 tptr, nt, 0 if message_mode == "dense" else 1,
                                 0 if softmax_mode == "twopass" else 1, float(chi),
                                 1 if score_mode == "nonlinear" else 0, _d(out))
    if rc != 0:
        raise ValueError("oracle rejected the configuration")
    return out


def cap_neighbors(pos, offsets, idx, K, translation=None):
    """Neighbour cap (the max_neighbors setting of the paper's model table): of every atom's neighbours keep the K
    nearest.  Distances are compared through the binary32 d^2 of the cutoff predicate ((dx*dx + dy*dy) + dz*dz, every
    operation rounded to binary32), ties go to the lower atom index.  Returns (offsets, idx), rows in atom order.
    translation: None, or [E][3] lattice translations of the neighbours' periodic images (pos is then the folded
    positions); a third array, the kept edges' positions in the input list, is returned as well."""
    p = np.asarray(pos, dtype=np.float32)
    new_off = np.zeros(len(offsets), dtype=np.int64)
    rows, kept = [], []
    for i in range(len(offsets) - 1):
        nb = np.asarray(idx[offsets[i]:offsets[i + 1]], dtype=np.int64)
        where = np.arange(offsets[i], offsets[i + 1])
        if len(nb) > K:
            pj = p[nb]
            if translation is not None:
                pj = pj + np.asarray(translation[offsets[i]:offsets[i + 1]], dtype=np.float32)
            d = pj - p[i]
            d2 = (d[:, 0] * d[:, 0] + d[:, 1] * d[:, 1]) + d[:, 2] * d[:, 2]
            assert d2.dtype == np.float32
            keep = np.lexsort((nb, d2))[:K]
            keep = keep[np.argsort(nb[keep])]
            nb, where = nb[keep], where[keep]
        rows.append(nb.astype(np.int32))
        kept.append(where)
        new_off[i + 1] = new_off[i] + len(nb)
    new_idx = (np.concatenate(rows) if rows else np.zeros(0, dtype=np.int32)).astype(np.int32)
    if translation is None:
        return new_off, new_idx
    return new_off, new_idx, (np.concatenate(kept) if kept else np.zeros(0, dtype=np.int64)).astype(np.int64)
