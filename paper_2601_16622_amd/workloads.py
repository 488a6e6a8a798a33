"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and lays out arrays: it holds none of the operator's arithmetic
and is the one module that both the HIP path's callers and the CPU oracle's callers read inputs from.
The molecular systems are stand-ins with the shapes of the paper's workloads (small organic molecules,
larger dense clusters with tens of neighbours inside a 6 Angstrom cutoff, and uniform-density boxes of
10^4..10^5 atoms for the scaling runs); no dataset item is reproduced.

Every generator returns a dict:
  cfg      dict(L, C, H, B, lf, cutoff, dtype)   dtype in {"f32", "bf16"}
  pos      float32 [N][3]
  seg      int32 [S+1]        segment offsets (one segment per independent system)
  h        float32 [N][(L+1)^2][C]   (for dtype "bf16": values already rounded to bfloat16)
  weights  dict(WQ1, WQ2, WK1, WK2, WV float32 [L+1][C][C] (out, in; bf16-rounded when dtype is bf16),
                Wb float32 [H][B], w_path float32 [L+1][L+1] indexed [l_in][l_out])
"""
import numpy as np

ELEMENT_PROBS = np.array([0.50, 0.30, 0.08, 0.08, 0.04 / 3, 0.04 / 3, 0.04 / 3])  # H C N O F S Cl


def round_to_bf16(x):
    """Round float32 values to the nearest bfloat16 (ties to even); result is float32 holding those values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


class _Grid:
    """Hash grid of edge `sep` used to reject points closer than `sep` to an accepted one."""

    def __init__(self, sep):
        self.sep = sep
        self.cells = {}

    def _key(self, p):
        return (int(np.floor(p[0] / self.sep)), int(np.floor(p[1] / self.sep)), int(np.floor(p[2] / self.sep)))

    def ok(self, p):
        kx, ky, kz = self._key(p)
        s2 = self.sep * self.sep
        for dx in (-1, 0, 1):
            for dy in (-1, 0, 1):
                for dz in (-1, 0, 1):
                    for q in self.cells.get((kx + dx, ky + dy, kz + dz), ()):
                        if (p[0] - q[0]) ** 2 + (p[1] - q[1]) ** 2 + (p[2] - q[2]) ** 2 < s2:
                            return False
        return True

    def add(self, p):
        self.cells.setdefault(self._key(p), []).append((float(p[0]), float(p[1]), float(p[2])))


def dart_throw_box(rng, n, side, min_sep=0.9, origin=(0.0, 0.0, 0.0)):
    """n points uniform in a cube of edge `side`, each at least min_sep from all others."""
    grid = _Grid(min_sep)
    out = np.empty((n, 3))
    k = 0
    while k < n:
        cand = rng.uniform(0.0, side, size=(max(256, n - k), 3))
        for p in cand:
            if grid.ok(p):
                grid.add(p)
                out[k] = p
                k += 1
                if k == n:
                    break
    return (out + np.asarray(origin)).astype(np.float32)


def bonded_cluster(rng, n, bond=(1.0, 1.6), min_sep=0.9):
    """Grow a molecule-like cluster: each new atom is bonded to a random earlier one."""
    grid = _Grid(min_sep)
    pts = [np.zeros(3)]
    grid.add(pts[0])
    while len(pts) < n:
        base = pts[rng.integers(len(pts))]
        u = rng.normal(size=3)
        u /= np.linalg.norm(u)
        p = base + u * rng.uniform(bond[0], bond[1])
        if grid.ok(p):
            grid.add(p)
            pts.append(p)
    return np.asarray(pts, dtype=np.float32)


def _weights(rng, L, C, H, B, dtype):
    lim = np.sqrt(6.0 / (2 * C))
    w = {}
    for name in ("WQ1", "WQ2", "WK1", "WK2", "WV"):
        x = rng.uniform(-lim, lim, size=(L + 1, C, C)).astype(np.float32)
        w[name] = round_to_bf16(x) if dtype == "bf16" else x
    w["Wb"] = (rng.normal(size=(H, B)) / np.sqrt(B)).astype(np.float32)
    w["w_path"] = rng.uniform(0.5, 1.5, size=(L + 1, L + 1)).astype(np.float32)
    return w


def _features(rng, N, L, C, dtype, elements=None):
    n = (L + 1) ** 2
    h = rng.normal(size=(N, n, C)).astype(np.float32)
    if elements is not None:
        table = rng.normal(size=(len(ELEMENT_PROBS), C)).astype(np.float32)
        h[:, 0, :] = table[elements]
    return round_to_bf16(h) if dtype == "bf16" else h


def _pack(cfg, pos_list, rng, elements=True):
    sizes = [p.shape[0] for p in pos_list]
    seg = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    pos = np.concatenate(pos_list, axis=0).astype(np.float32)
    N = pos.shape[0]
    el = rng.choice(len(ELEMENT_PROBS), size=N, p=ELEMENT_PROBS) if elements else None
    h = _features(rng, N, cfg["L"], cfg["C"], cfg["dtype"], el)
    w = _weights(rng, cfg["L"], cfg["C"], cfg["H"], cfg["B"], cfg["dtype"])
    return {"cfg": cfg, "pos": pos, "seg": seg, "h": h, "weights": w, "elements": el}


def tiny(seed=0):
    rng = np.random.default_rng(seed)
    cfg = dict(L=1, C=16, H=2, B=8, lf=1, cutoff=5.0, dtype="f32")
    return _pack(cfg, [dart_throw_box(rng, 64, 8.0)], rng, elements=False)


def small_molecules(seed=0, n_mol=64, lo=10, hi=60):
    rng = np.random.default_rng(seed)
    cfg = dict(L=2, C=128, H=8, B=8, lf=1, cutoff=5.0, dtype="f32")
    sizes = rng.integers(lo, hi + 1, size=n_mol)
    mols = [bonded_cluster(rng, int(s)) + rng.uniform(-20, 20, size=3).astype(np.float32) for s in sizes]
    return _pack(cfg, mols, rng)


def large_molecules(seed=0, n_sys=16, lo=150, hi=350):
    rng = np.random.default_rng(seed)
    cfg = dict(L=4, C=128, H=8, B=8, lf=1, cutoff=6.0, dtype="bf16")
    sizes = rng.integers(lo, hi + 1, size=n_sys)
    systems = [dart_throw_box(rng, int(s), (s / 0.1) ** (1.0 / 3.0), origin=rng.uniform(-30, 30, size=3))
               for s in sizes]
    return _pack(cfg, systems, rng)


def box(n_atoms, seed=0, L=4, C=128, H=8, B=8, cutoff=6.0, dtype="bf16", density=0.1):
    """One non-periodic cubic box of n_atoms at the given number density (atoms per cubic Angstrom)."""
    rng = np.random.default_rng(seed)
    cfg = dict(L=L, C=C, H=H, B=B, lf=1, cutoff=cutoff, dtype=dtype)
    side = (n_atoms / density) ** (1.0 / 3.0)
    return _pack(cfg, [dart_throw_box(rng, n_atoms, side)], rng)


def fcc_subsample(n_atoms, seed=0, a=3.8, L=4, C=128, H=8, B=8, cutoff=6.0, dtype="bf16"):
    """The system recipe of the paper's inference-scaling experiment (App. "System generation"): the smallest cubic
    FCC supercell with lattice constant a that holds n_atoms sites, n_atoms of them drawn without replacement; no
    periodic images.  A full lattice has 54 sites inside 6 A of a site (12 + 6 + 24 + 12); many pairs are exactly
    equidistant, which exercises the tie rule of the neighbour cap."""
    rng = np.random.default_rng(seed)
    cfg = dict(L=L, C=C, H=H, B=B, lf=1, cutoff=cutoff, dtype=dtype)
    nc = 1
    while 4 * nc ** 3 < n_atoms:
        nc += 1
    cell = np.stack(np.meshgrid(np.arange(nc), np.arange(nc), np.arange(nc), indexing="ij"), -1).reshape(-1, 3)
    basis = np.array([[0.0, 0.0, 0.0], [0.0, 0.5, 0.5], [0.5, 0.0, 0.5], [0.5, 0.5, 0.0]])
    sites = ((cell[:, None, :] + basis[None, :, :]) * a).reshape(-1, 3)
    keep = rng.choice(len(sites), n_atoms, replace=False)
    return _pack(cfg, [sites[np.sort(keep)].astype(np.float32)], rng)


def periodic_boxes(n_atoms=(600,), seed=0, L=4, C=128, H=8, B=8, cutoff=6.0, dtype="bf16", density=0.1, open_axes=()):
    """Periodic systems (bulk simulation cells, as in the paper's condensed-phase runs, Sec. 4.3): one orthorhombic
    box per segment at the given number density, edge lengths in the ratio 1 : 1.1 : 0.95, atoms thrown so that
    periodic images keep the minimum separation too; coordinates are then displaced by whole box lengths for a
    tenth of the atoms, so callers see coordinates outside [0, len) as an MD run produces them.  Axes listed in
    open_axes are not periodic (a slab).  The dict carries "box": float32 [S][3], 0 on an open axis."""
    rng = np.random.default_rng(seed)
    cfg = dict(L=L, C=C, H=H, B=B, lf=1, cutoff=cutoff, dtype=dtype)
    pos_list, boxes = [], []
    for n in n_atoms:
        base = (n / density / (1.1 * 0.95)) ** (1.0 / 3.0)
        lens = np.array([base, 1.1 * base, 0.95 * base]).astype(np.float32)
        lens = np.maximum(lens, np.float32(3.0 * cutoff * 1.001))
        grid = _Grid(0.9)
        pts = np.empty((n, 3))
        k = 0
        while k < n:
            for u in rng.uniform(0.0, 1.0, size=(max(256, n - k), 3)):
                p = 0.45 + u * (lens - 0.9)
                if grid.ok(p):
                    grid.add(p)
                    pts[k] = p
                    k += 1
                    if k == n:
                        break
        moved = rng.random(n) < 0.1
        hop = rng.integers(-2, 3, size=(n, 3)) * lens[None, :]
        for ax in open_axes:
            hop[:, ax] = 0.0
        pts = pts + np.where(moved[:, None], hop, 0.0)
        bx = lens.copy()
        for ax in open_axes:
            bx[ax] = 0.0
        pos_list.append(pts.astype(np.float32))
        boxes.append(bx)
    out = _pack(cfg, pos_list, rng)
    out["box"] = np.stack(boxes).astype(np.float32)
    return out


def periodic_fcc(nc=5, seed=0, a=3.8, L=4, C=128, H=8, B=8, cutoff=6.0, dtype="bf16"):
    """A full periodic FCC crystal of nc^3 conventional cells (lattice constant a): every atom has the same
    environment, 54 neighbours inside 6 A for a = 3.8 (shells of 12, 6, 24 and 12; the next shell is at 6.008)."""
    rng = np.random.default_rng(seed)
    cfg = dict(L=L, C=C, H=H, B=B, lf=1, cutoff=cutoff, dtype=dtype)
    cell = np.stack(np.meshgrid(np.arange(nc), np.arange(nc), np.arange(nc), indexing="ij"), -1).reshape(-1, 3)
    basis = np.array([[0.0, 0.0, 0.0], [0.0, 0.5, 0.5], [0.5, 0.0, 0.5], [0.5, 0.5, 0.0]])
    sites = ((cell[:, None, :] + basis[None, :, :]) * a).reshape(-1, 3)
    out = _pack(cfg, [sites.astype(np.float32)], rng)
    out["box"] = np.full((1, 3), nc * a, dtype=np.float32)
    return out


def scaling_point(seed=0):
    return box(10_000, seed)


def by_name(name, seed=0):
    if name == "tiny":
        return tiny(seed)
    if name == "small":
        return small_molecules(seed)
    if name == "large":
        return large_molecules(seed)
    if name == "scaling":
        return scaling_point(seed)
    if name.startswith("box"):
        return box(int(name[3:]), seed)
    if name.startswith("fcc"):
        return fcc_subsample(int(name[3:]), seed)
    if name.startswith("pbox"):
        return periodic_boxes((int(name[4:]),), seed)
    raise KeyError(name)
