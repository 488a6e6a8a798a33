"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header declares,
validates configurations, reports closed-form workspace sizes and rejects bad arguments before launching."""
import ctypes
import os
import re

import numpy as np

import pytest

from paper_2601_16622_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2601_16622_amd import build
        build.build(verbose=False)
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "e2f.h")).read()
    declared = set(re.findall(r"\b(e2f_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    texts = {B.status_string(c) for c in range(7)}
    assert len(texts) == 7 and "ok" in texts


@pytest.mark.parametrize("kw,code", [
    (dict(L_max=-1), 1), (dict(C=0), 1), (dict(H=3), 1), (dict(B=0), 1), (dict(cutoff=0.0), 1),
    (dict(cutoff=float("nan")), 1), (dict(feat_dtype=7), 1), (dict(L_max=0, lf=1), 1),
    (dict(L_max=5), 2), (dict(lf=3, L_max=4), 2), (dict(lf=2, L_max=1), 1), (dict(C=24, H=2), 2), (dict(C=320, H=8), 2), (dict(C=16, H=2, feat_dtype=1), 2),
    (dict(attention=4), 1), (dict(attention=-1), 1), (dict(flags=64), 1),
    (dict(attention=1, C=64, H=8), 2),      # the tile kernels want heads of 16 channels
    (dict(attention=1, lf=2), 2),           # ... and the degree-1 filter
    (dict(attention=2, feat_dtype=0), 2),   # the per-pair matrix-core kernel wants bf16 features
])
def test_create_rejects_bad_configurations(lib, kw, code):
    base = dict(L_max=2, C=128, H=8, B=8, lf=1, cutoff=5.0, feat_dtype=0, attention=0, flags=0)
    base.update(kw)
    cfg = B.Config(*[base[k] for k in ("L_max", "C", "H", "B", "lf", "cutoff", "feat_dtype", "attention", "flags")])
    ctx = ctypes.c_void_p()
    assert lib.e2f_create(ctypes.byref(cfg), ctypes.byref(ctx)) == code
    assert not ctx.value


def test_workspace_sizes_are_linear_in_N(lib):
    ctx = B.e2f_create(4, 128, 8, 8, 1, 6.0, "bf16")
    try:
        sizes = [B.e2f_attn_workspace_bytes(ctx, N) for N in (10_000, 20_000, 40_000)]
        # per atom (tile kernel): sorted position 16 B, q and k binary16 with 96 features per head (80 padded to a
        # multiple of 32), v bf16 [25][128]; per tile of 16 atoms a candidate list of 192 entries (header 16 B,
        # entry 4 B, four slot positions 64 B, pair mask 8 B)
        per_atom = 16 + 2 * 8 * 96 * 2 + 25 * 128 * 2 + (16 + 192 * (4 + 64 + 8)) // 16
        assert abs((sizes[1] - sizes[0]) - 10_000 * per_atom) <= 2048
        assert abs((sizes[2] - sizes[1]) - 20_000 * per_atom) <= 2048
        c = [B.e2f_cells_workspace_bytes(ctx, N, 4) for N in (1000, 2000, 3000)]
        assert abs((c[2] - c[1]) - (c[1] - c[0])) <= 4096
        assert B.e2f_attn_workspace_bytes(ctx, -1) == 0
    finally:
        B.e2f_destroy(ctx)


def test_entry_points_reject_bad_arguments_before_launching(lib):
    ctx = B.e2f_create(1, 16, 2, 8, 1, 5.0, "f32")
    try:
        cells = ctypes.c_void_p()
        null = ctypes.c_void_p(0)
        # null positions with N > 0, negative N, unaligned / too small workspace
        assert lib.e2f_build_cells(ctx, null, null, 4, 1, null, 0, ctypes.byref(cells), null) == 1
        assert lib.e2f_build_cells(ctx, null, null, -1, 1, null, 0, ctypes.byref(cells), null) == 1
        fake = ctypes.c_void_p(4096)
        assert lib.e2f_build_cells(ctx, fake, fake, 4, 1, ctypes.c_void_p(4096 + 8), 1 << 20, ctypes.byref(cells), null) == 1
        assert lib.e2f_build_cells(ctx, fake, fake, 4, 1, fake, 16, ctypes.byref(cells), null) == 3
        # an empty problem is valid and launches nothing
        assert lib.e2f_build_cells(ctx, null, null, 0, 0, null, 0, ctypes.byref(cells), null) == 0
        w = B.Weights(*([0] * 7))
        assert lib.e2f_attn_forward(ctx, cells, null, null, null, 0, 0, ctypes.byref(w), null, null, 0, null) == 0
        assert lib.e2f_attn_forward(ctx, cells, null, null, null, 5, 1, ctypes.byref(w), null, null, 0, null) == 1
        assert lib.e2f_attn_forward(ctx, null, null, null, null, 0, 0, ctypes.byref(w), null, null, 0, null) == 1
        lib.e2f_cells_destroy(cells)
    finally:
        B.e2f_destroy(ctx)


def test_periodic_cells_validate_the_box_on_the_host(lib):
    """A periodic edge must hold three cell edges (3 * 1.0001 * cutoff) and be finite; entries <= 0 or NaN mean an
    open axis.  All of this is decided before anything is launched."""
    ctx = B.e2f_create(1, 16, 2, 8, 1, 5.0, "f32")
    try:
        cells = ctypes.c_void_p()
        null, fake = ctypes.c_void_p(0), ctypes.c_void_p(4096)

        def build(box, N=4, ws=fake, ws_bytes=16):
            b = np.ascontiguousarray(box, dtype=np.float32)
            return lib.e2f_build_cells_periodic(ctx, fake, fake, N, 1, ctypes.c_void_p(b.ctypes.data), ws, ws_bytes,
                                                ctypes.byref(cells), null)
        assert build([[15.0, 40.0, 40.0]]) == 2            # 15 < 15.0015
        assert build([[40.0, 40.0, np.inf]]) == 2
        assert build([[15.002, 0.0, -3.0]]) == 3           # valid box: the next check (workspace size) answers
        assert build([[np.nan, 0.0, 0.0]]) == 3            # no periodic axis at all
        assert build([[15.002, 15.002, 15.002]], ws=ctypes.c_void_p(4096 + 8), ws_bytes=1 << 20) == 1
        # NULL box: the open-boundary call
        assert lib.e2f_build_cells_periodic(ctx, null, null, 0, 0, null, null, 0, ctypes.byref(cells), null) == 0
        lib.e2f_cells_destroy(cells)
    finally:
        B.e2f_destroy(ctx)


def test_factorized_entry_point_sizes_and_limits(lib):
    """Three more fp32 [N][n][C] arrays on top of the untiled attention workspace; lf != 1 and head widths that are
    not a power of two <= 64 are refused before anything is launched."""
    ctx = B.e2f_create(4, 128, 8, 8, 1, 6.0, "bf16")
    try:
        s = [B.e2f_attn_factorized_workspace_bytes(ctx, N) for N in (10_000, 20_000)]
        per_atom = 16 + 2 * 5 * 128 * 4 + 25 * 128 * 2 + 3 * 25 * 128 * 4
        assert abs((s[1] - s[0]) - 10_000 * per_atom) <= 4096
        assert B.e2f_attn_factorized_workspace_bytes(ctx, -1) == 0
        cells = ctypes.c_void_p()
        null = ctypes.c_void_p(0)
        assert lib.e2f_build_cells(ctx, null, null, 0, 0, null, 0, ctypes.byref(cells), null) == 0
        w = B.Weights(*([0] * 7))
        assert lib.e2f_attn_forward_factorized(ctx, cells, null, null, null, 0, 0, ctypes.byref(w), null, null, 0, null) == 0
        assert lib.e2f_attn_forward_factorized(ctx, cells, null, null, null, 5, 1, ctypes.byref(w), null, null, 0, null) == 1
        lib.e2f_cells_destroy(cells)
    finally:
        B.e2f_destroy(ctx)
    for kw in (dict(lf=2), dict(lf=0), dict(C=192, H=1), dict(C=256, H=2)):
        a = dict(L_max=2, C=64, H=4, B=8, lf=1)
        a.update(kw)
        ctx = B.e2f_create(a["L_max"], a["C"], a["H"], a["B"], a["lf"], 5.0, "f32")
        try:
            w = B.Weights(*([0] * 7))
            assert lib.e2f_attn_forward_factorized(ctx, None, None, None, None, 0, 0, ctypes.byref(w), None, None, 0, None) == 2
        finally:
            B.e2f_destroy(ctx)


def test_nonlinear_entry_point_sizes_and_limits(lib):
    """The plain-layout attention workspace plus W_Q1 h as one more [N][n][C] array of the feature type; heads wider
    than a wave are refused before anything is launched."""
    ctx = B.e2f_create(4, 128, 8, 8, 1, 6.0, "bf16")
    try:
        s = [B.e2f_attn_nonlinear_workspace_bytes(ctx, N) for N in (10_000, 20_000)]
        per_atom = 16 + 2 * 5 * 128 * 4 + 2 * 25 * 128 * 2
        assert abs((s[1] - s[0]) - 10_000 * per_atom) <= 4096
        assert B.e2f_attn_nonlinear_workspace_bytes(ctx, -1) == 0
        cells = ctypes.c_void_p()
        null = ctypes.c_void_p(0)
        assert lib.e2f_build_cells(ctx, null, null, 0, 0, null, 0, ctypes.byref(cells), null) == 0
        w = B.Weights(*([0] * 7))
        assert lib.e2f_attn_forward_nonlinear(ctx, cells, null, null, null, 0, 0, ctypes.byref(w), null, null, 0, null) == 0
        assert lib.e2f_attn_forward_nonlinear(ctx, cells, null, null, null, 5, 1, ctypes.byref(w), null, null, 0, null) == 1
        assert lib.e2f_attn_forward_nonlinear(None, cells, null, null, null, 0, 0, ctypes.byref(w), null, null, 0, null) == 1
        lib.e2f_cells_destroy(cells)
    finally:
        B.e2f_destroy(ctx)
    for kw in (dict(C=128, H=1), dict(C=256, H=2)):
        a = dict(L_max=2, C=64, H=4, B=8, lf=1)
        a.update(kw)
        ctx = B.e2f_create(a["L_max"], a["C"], a["H"], a["B"], a["lf"], 5.0, "f32")
        try:
            w = B.Weights(*([0] * 7))
            assert lib.e2f_attn_forward_nonlinear(ctx, None, None, None, None, 0, 0, ctypes.byref(w), None, None, 0, None) == 2
        finally:
            B.e2f_destroy(ctx)


def test_backward_entry_point_sizes_and_limits(lib):
    """Per-atom kernels: two [N][H] statistics arrays, the partial sums of the weight gradients and the axis operators
    on top of the untiled attention workspace.  Tile form (where the forward pass runs on the tile kernels): the tile
    layouts of q, k, v, the candidate lists, and the operands the forward pass does not keep (q grouped, q and k with
    four slots per lane, rows of v and dL/d out, dL/d out in v's layout, statistics, partial position gradients).
    The degree-1 filter and power-of-two head widths up to 64 only; an empty problem is valid; null gradients are not."""
    stats = 2 * 8 * 4 + 8 * 8 * 4 + 32 * 4
    per_atom_plain = 16 + 2 * 5 * 128 * 4 + 25 * 128 * 2 + stats
    qk = 8 * 96 * 2
    per_atom_tile = (16 + 2 * qk + 8 * 25 * 16 * 2 + (16 + 192 * (4 + 64 + 8)) // 16 + stats
                     + 3 * qk + 2 * 8 * 416 * 2 + 8 * 25 * 16 * 2 + 8 * 8 + 2 * 8 * 3 * 4
                     + (8 * 8 * 4 + 8 * 32 * 4) // 16)   # per tile of 16 atoms: partial sums of dL/dWb and dL/dw_path
    ctx = B.e2f_create(4, 128, 8, 8, 1, 6.0, "bf16", attention="valu")
    try:
        s = [B.e2f_attn_backward_workspace_bytes(ctx, N) for N in (10_000, 20_000)]
        assert abs((s[1] - s[0]) - 10_000 * per_atom_plain) <= 4096
    finally:
        B.e2f_destroy(ctx)
    ctx = B.e2f_create(4, 128, 8, 8, 1, 6.0, "bf16")
    try:
        s = [B.e2f_attn_backward_workspace_bytes(ctx, N) for N in (10_000, 20_000)]
        per_atom = per_atom_tile
        assert abs((s[1] - s[0]) - 10_000 * per_atom) <= 4096
        assert B.e2f_attn_backward_workspace_bytes(ctx, -1) == 0
        sw = [B.e2f_attn_backward_weights_workspace_bytes(ctx, N) for N in (10_000, 20_000)]
        assert abs((sw[1] - sw[0]) - 10_000 * (per_atom + 5 * 25 * 128 * 4)) <= 4096
        assert sw[0] - s[0] >= 5 * 10_000 * 25 * 128 * 4 + 8 * 25 * 5 * 128 * 128 * 4
        cells = ctypes.c_void_p()
        null = ctypes.c_void_p(0)
        assert lib.e2f_build_cells(ctx, null, null, 0, 0, null, 0, ctypes.byref(cells), null) == 0
        w = B.Weights(*([0] * 7))

        def call(N, S, ptr):
            return lib.e2f_attn_backward(ctx, cells, ptr, ptr, ptr, N, S, ctypes.byref(w), ptr, ptr, ptr, ptr, ptr, ptr,
                                         null, null, null, null, ptr, 0, null)
        assert call(0, 0, null) == 0
        assert call(5, 1, null) == 1
        lib.e2f_cells_destroy(cells)
    finally:
        B.e2f_destroy(ctx)
    for kw in (dict(lf=2), dict(lf=0), dict(C=192, H=1), dict(C=96 * 2, H=2)):
        a = dict(L_max=2, C=64, H=4, B=8, lf=1)
        a.update(kw)
        ctx = B.e2f_create(a["L_max"], a["C"], a["H"], a["B"], a["lf"], 5.0, "f32")
        try:
            w = B.Weights(*([0] * 7))
            assert lib.e2f_attn_backward(ctx, None, None, None, None, 0, 0, ctypes.byref(w), None, None, None, None, None,
                                         None, None, None, None, None, None, 0, None) == 2
        finally:
            B.e2f_destroy(ctx)


def test_cap_and_table_entry_points_reject_bad_arguments(lib):
    ctx = B.e2f_create(1, 16, 2, 8, 1, 5.0, "f32")
    try:
        cells = ctypes.c_void_p()
        null = ctypes.c_void_p(0)
        assert lib.e2f_build_cells(ctx, null, null, 0, 0, null, 0, ctypes.byref(cells), null) == 0
        w = B.Weights(*([0] * 7))
        # an empty problem is fine; a cap or a table width of zero is not; a null table with atoms is not
        assert lib.e2f_attn_forward_capped(ctx, cells, null, null, null, 0, 0, ctypes.byref(w), 8, null, null, 0, null) == 0
        assert lib.e2f_attn_forward_capped(ctx, cells, null, null, null, 0, 0, ctypes.byref(w), 0, null, null, 0, null) == 1
        assert lib.e2f_attn_forward_table(ctx, cells, null, null, null, 0, 0, ctypes.byref(w), null, 0, null, null, 0, null) == 1
        assert lib.e2f_attn_forward_table(ctx, cells, null, null, null, 5, 1, ctypes.byref(w), null, 4, null, null, 0, null) == 1
        assert lib.e2f_build_neighbor_table(ctx, cells, null, 0, 0, null, null, null) == 1
        assert lib.e2f_build_neighbor_table(ctx, cells, null, 3, 4, null, null, null) == 1   # N does not match the cells
        n = 10_000
        assert B.e2f_attn_capped_workspace_bytes(ctx, n) - B.e2f_attn_workspace_bytes(ctx, n) == 2 * ((n * 4 + 255) // 256 * 256)
        assert B.e2f_attn_table_workspace_bytes(ctx, n) >= B.e2f_attn_workspace_bytes(ctx, n)
        lib.e2f_cells_destroy(cells)
    finally:
        B.e2f_destroy(ctx)


def test_axis_operator_pattern_matches_the_dense_definition():
    """The compile-time sparsity pattern of the three axis operators G_mu = (.) (x) R^(1)(e_mu) used by the tile kernel
    is exactly the non-zero pattern of the oracle's dense Clebsch-Gordan message for r = e_mu (216 entries, L_max = 4)."""
    import re
    import oracle as O
    txt = open(os.path.join(ROOT, "paper_2601_16622_amd", "csrc", "e2f_axis_pattern.h")).read()
    rows = re.findall(r"\{((?:0x[0-9a-f]+u,? ?)+)\}", txt)
    mask = [[int(x.strip().rstrip("u"), 16) for x in r.split(",")] for r in rows]
    assert len(mask) == 3 and all(len(r) == 25 for r in mask)
    w = np.random.default_rng(0).uniform(0.5, 1.5, (5, 5))
    total = 0
    for mu in range(3):
        for xi in range(25):
            v = np.zeros((25, 1))
            v[xi] = 1.0
            col = np.asarray(O.message(4, 1, w, v, np.eye(3)[mu], mode="dense")).reshape(25)
            for xo in range(25):
                assert bool((mask[mu][xo] >> xi) & 1) == bool(abs(col[xo]) > 1e-12), (mu, xo, xi)
                total += (mask[mu][xo] >> xi) & 1
    assert total == 216


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2601_16622_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "e2fo_" not in text, f
