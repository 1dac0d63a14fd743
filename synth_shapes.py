"""Seeded synthetic surface-voxel shapes, features, weights and gradients.

Input generators only.  Nothing here belongs to the method under test (no
hashing, no lookup, no convolution, no pooling): the functions produce voxel
coordinates of thin surface shells, per-voxel feature rows, weight tensors and
upstream gradients.  Both the CPU oracle's tests and the GPU path's tests,
the smoke check and the benchmark draw their inputs from here, so that the two
implementations always see the same numbers.

Shapes stand in for the surface voxelisations of mesh data sets the paper
trains on (Section 5: ModelNet40, ShapeNet Core55), which are not available:
like those they are two-dimensional surfaces embedded in a cube (n ~ c * u^2
occupied voxels at resolution u), possibly with several components.

Conventions
-----------
* coordinates are int32 (x, y, z) in [0, u); within one shape they are sorted
  by the linear index (x*u + y)*u + z, ascending (what numpy.nonzero yields);
* a batch is (coords [N,3], model_offsets [b+1] int64), shapes concatenated;
* feature rows are voxel-major: X[N, C];
* weights are W[27, C_in, C_out] with tap k = (dx+1)*9 + (dy+1)*3 + (dz+1).
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# signed distance functions of the three primitives (negative inside)
# ----------------------------------------------------------------------------


def _sdf_sphere(p, c, r):
    return np.sqrt(((p - c) ** 2).sum(-1)) - r


def _sdf_box(p, c, h):
    q = np.abs(p - c) - h
    outside = np.sqrt((np.maximum(q, 0.0) ** 2).sum(-1))
    inside = np.minimum(q.max(-1), 0.0)
    return outside + inside


def _sdf_torus(p, c, R, r):
    d = p - c
    ring = np.sqrt(d[..., 0] ** 2 + d[..., 1] ** 2) - R
    return np.sqrt(ring ** 2 + d[..., 2] ** 2) - r


def _sdf_prim(p, prim):
    kind = prim[0]
    if kind == "sphere":
        return _sdf_sphere(p, prim[1], prim[2])
    if kind == "box":
        return _sdf_box(p, prim[1], prim[2])
    return _sdf_torus(p, prim[1], prim[2], prim[3])


def _prim_bbox(prim, u):
    kind, c = prim[0], prim[1]
    if kind == "sphere":
        ext = np.full(3, prim[2])
    elif kind == "box":
        ext = np.asarray(prim[2], dtype=np.float64)
    else:
        ext = np.array([prim[2] + prim[3], prim[2] + prim[3], prim[3]])
    lo = np.clip(np.floor(c - ext - 1.0).astype(np.int64), 0, u)
    hi = np.clip(np.ceil(c + ext + 1.0).astype(np.int64) + 1, 0, u)
    return lo, hi


def random_primitives(rng, u, n_min=1, n_max=4):
    """1..4 (or n_min..n_max) random primitives with all lengths scaled by u/64."""
    s = u / 64.0
    count = int(rng.integers(n_min, n_max + 1))
    prims = []
    for _ in range(count):
        kind = ("sphere", "box", "torus")[int(rng.integers(0, 3))]
        c = rng.uniform(16.0, 48.0, size=3) * s
        if kind == "sphere":
            prims.append((kind, c, float(rng.uniform(6.0, 20.0)) * s))
        elif kind == "box":
            prims.append((kind, c, rng.uniform(4.0, 16.0, size=3) * s))
        else:
            prims.append((kind, c, float(rng.uniform(8.0, 18.0)) * s,
                          float(rng.uniform(2.0, 5.0)) * s))
    return prims


def _inside_mask(prims, u):
    """Boolean u^3 grid: voxel centre (i+.5, j+.5, k+.5) inside the union."""
    inside = np.zeros((u, u, u), dtype=bool)
    for prim in prims:
        lo, hi = _prim_bbox(prim, u)
        if np.any(hi <= lo):
            continue
        # evaluate slab by slab to bound temporary memory at high resolution
        ys = np.arange(lo[1], hi[1], dtype=np.float32) + 0.5
        zs = np.arange(lo[2], hi[2], dtype=np.float32) + 0.5
        step = max(1, int(4_000_000 // max(1, ys.size * zs.size)))
        for x0 in range(int(lo[0]), int(hi[0]), step):
            x1 = min(int(hi[0]), x0 + step)
            xs = np.arange(x0, x1, dtype=np.float32) + 0.5
            g = np.stack(np.meshgrid(xs, ys, zs, indexing="ij"), axis=-1)
            prim32 = tuple(np.asarray(a, dtype=np.float32) if not isinstance(a, str) else a
                           for a in prim)
            sd = _sdf_prim(g, prim32)
            inside[x0:x1, lo[1]:hi[1], lo[2]:hi[2]] |= sd < 0
    return inside


def _erode6(mask):
    """Voxels whose six face neighbours are all set (off-grid counts as unset)."""
    e = mask.copy()
    for ax in range(3):
        sl_lo = [slice(None)] * 3
        sl_hi = [slice(None)] * 3
        sl_lo[ax] = slice(0, -1)
        sl_hi[ax] = slice(1, None)
        nb = np.zeros_like(mask)
        nb[tuple(sl_lo)] = mask[tuple(sl_hi)]      # neighbour at +1
        e &= nb
        nb = np.zeros_like(mask)
        nb[tuple(sl_hi)] = mask[tuple(sl_lo)]      # neighbour at -1
        e &= nb
    return e


def _dilate6(mask):
    d = mask.copy()
    for ax in range(3):
        sl_lo = [slice(None)] * 3
        sl_hi = [slice(None)] * 3
        sl_lo[ax] = slice(0, -1)
        sl_hi[ax] = slice(1, None)
        d[tuple(sl_lo)] |= mask[tuple(sl_hi)]
        d[tuple(sl_hi)] |= mask[tuple(sl_lo)]
    return d


def shell_from_primitives(prims, u, thick=False):
    """Surface shell of the union of primitives on a u^3 grid.

    thin  : inside voxels with at least one of the 6 face neighbours outside
            (off-grid counts as outside) -- one voxel thick;
    thick : the thin shell plus the outside voxels that face-touch the solid
            -- about two voxels thick (used for the highest resolution).
    Returns int32 coords [n,3] sorted by (x*u+y)*u+z.
    """
    inside = _inside_mask(prims, u)
    shell = inside & ~_erode6(inside)
    if thick:
        shell |= (~inside) & _dilate6(inside)
    xs, ys, zs = np.nonzero(shell)
    return np.stack([xs, ys, zs], axis=1).astype(np.int32)


def sdf_normals(prims, coords):
    """Unit normals: normalised central-difference gradient of the union SDF
    (min over primitives) at the voxel centres; float64 [n,3]."""
    p = coords.astype(np.float64) + 0.5

    def sdf(q):
        d = _sdf_prim(q, prims[0])
        for prim in prims[1:]:
            d = np.minimum(d, _sdf_prim(q, prim))
        return d

    g = np.empty_like(p)
    h = 0.5
    for ax in range(3):
        e = np.zeros(3)
        e[ax] = h
        g[:, ax] = (sdf(p + e) - sdf(p - e)) / (2 * h)
    nrm = np.sqrt((g ** 2).sum(-1, keepdims=True))
    g = np.where(nrm > 1e-12, g / np.maximum(nrm, 1e-12), np.array([0.0, 0.0, 1.0]))
    return g


# ----------------------------------------------------------------------------
# named workloads
# ----------------------------------------------------------------------------


def sphere_shell_32():
    """The single-shape case: 32^3 grid, sphere of radius 12 centred at
    (16,16,16); a voxel is occupied iff |dist(centre, sphere centre) - 12| < 0.87.
    Returns coords int32 [n,3] (sorted) and the unit outward normals float32 [n,3]."""
    u = 32
    ax = np.arange(u, dtype=np.float64) + 0.5
    g = np.stack(np.meshgrid(ax, ax, ax, indexing="ij"), axis=-1) - 16.0
    dist = np.sqrt((g ** 2).sum(-1))
    occ = np.abs(dist - 12.0) < 0.87
    xs, ys, zs = np.nonzero(occ)
    coords = np.stack([xs, ys, zs], axis=1).astype(np.int32)
    normals = (g[xs, ys, zs] / dist[xs, ys, zs][:, None]).astype(np.float32)
    return coords, normals


def primitive_batch(u, batch, seed_base, n_min=1, n_max=4, thick=False, with_normals=False):
    """Batch of random-primitive shells on a u^3 grid.

    Shape i is drawn from numpy.random.default_rng(seed_base + i).  Returns
    (coords int32 [N,3], model_offsets int64 [batch+1], normals float32 [N,3] or None).
    """
    all_c, all_n, offs = [], [], [0]
    for i in range(batch):
        rng = np.random.default_rng(seed_base + i)
        prims = random_primitives(rng, u, n_min, n_max)
        c = shell_from_primitives(prims, u, thick=thick)
        if c.shape[0] == 0:                      # cannot happen for the stated ranges
            c = np.array([[u // 2, u // 2, u // 2]], dtype=np.int32)
        all_c.append(c)
        if with_normals:
            all_n.append(sdf_normals(prims, c).astype(np.float32))
        offs.append(offs[-1] + c.shape[0])
    coords = np.concatenate(all_c, axis=0)
    normals = np.concatenate(all_n, axis=0) if with_normals else None
    return coords, np.asarray(offs, dtype=np.int64), normals


CONFIGS = {
    # id: (resolution, batch, lengths scale is u/64, primitives min..max, thick shell)
    2: dict(u=64, batch=32, n_min=1, n_max=4, thick=False),
    3: dict(u=128, batch=16, n_min=1, n_max=4, thick=False),
    4: dict(u=256, batch=8, n_min=1, n_max=4, thick=False),
    5: dict(u=512, batch=4, n_min=2, n_max=6, thick=True),
}


def config_batch(config, batch=None, u=None, with_normals=False):
    """Geometry of workload `config` (2..5); `batch`/`u` override for scaled-down tests.
    Seeds are 1000*config + shape index."""
    cfg = dict(CONFIGS[config])
    if batch is not None:
        cfg["batch"] = batch
    if u is not None:
        cfg["u"] = u
    return primitive_batch(cfg["u"], cfg["batch"], 1000 * config, cfg["n_min"], cfg["n_max"],
                           cfg["thick"], with_normals)


def normals_plus_one(normals):
    """4-channel input rows: unit normal and a constant occupancy channel."""
    n = normals.shape[0]
    return np.concatenate([normals.astype(np.float32), np.ones((n, 1), np.float32)], axis=1)


def gaussian(shape, std, seed):
    """float32 N(0, std^2) tensor from numpy.random.default_rng(seed)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(size=shape) * std).astype(np.float32)


def he_weights(c_in, c_out, seed):
    """W[27, c_in, c_out] ~ N(0, 2/(27 c_in)), float32."""
    return gaussian((27, c_in, c_out), float(np.sqrt(2.0 / (27.0 * c_in))), seed)


def to_bf16_grid(x):
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32.
    Pure bit arithmetic on the inputs; used so that both implementations start from
    identical bf16-representable numbers."""
    a = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (a >> 16) & 1
    a = (a + 0x7FFF + lsb) & 0xFFFF0000
    return a.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def bf16_bits(x):
    """uint16 bfloat16 bit patterns of values already on the bf16 grid."""
    a = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (a >> 16).astype(np.uint16).reshape(np.shape(x))
