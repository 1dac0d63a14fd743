"""Pins of the CPU oracle's hash construction and lookup against what the paper and
plain mathematics fix (CPU only).

Nothing here re-uses the oracle's own arithmetic: the checks are the printed values
of the worked 2-D example (Section 3.1), the size rules of Section 5.2, the validity
invariants of a perfect hash (Section 3.1), brute force through a dense index volume,
and numpy.cumsum for the prefix arrays of Section 3.2.
"""
import os

import numpy as np
import pytest

import synth_shapes as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def dense_index_volume(coords, u):
    vol = np.full((u, u, u), -1, np.int64)
    vol[coords[:, 0], coords[:, 1], coords[:, 2]] = np.arange(coords.shape[0])
    return vol


def numpy_lookup(L, v, P):
    """Independent vectorised restatement of the query protocol of Section 3.1 for
    in-grid positions P [k,3] of model v (used to cross-examine the oracle's tables)."""
    m, r = int(L.mbar[v]), int(L.rbar[v])
    P = np.asarray(P, np.int64)
    iphi = L.R[v] + ((P[:, 0] % r) * r + P[:, 1] % r) * r + P[:, 2] % r
    off = L.Phi[iphi].astype(np.int64)
    h = (P % m + off) % m
    s = L.M[v] + (h[:, 0] * m + h[:, 1]) * m + h[:, 2]
    ok = (L.H[s] != -1) & (L.T[s].astype(np.int64) == P).all(1)
    return np.where(ok, L.N[v] + L.H[s], -1), s


# --------------------------------------------------------------------------------------
# worked example and batch offsets
# --------------------------------------------------------------------------------------

def test_worked_2d_example(oracle):
    """Section 3.1 worked example, embedded as the z = 0 plane of a 3-D table: the
    oracle's Eq.1 must land on slot (1,0), read data index 3, accept the tag (3,1), and
    reject a query that lands on the redundant slot (2,1) or on a slot owned by another
    pixel."""
    g = _read_golden("psh_worked_example_2d.txt")
    m, r = g["m"][0], g["r"][0]
    qx, qy = g["query"]
    assert [qx % m, qy % m] == g["h0"] and [qx % r, qy % r] == g["h1"]
    H = np.full((m, m, m), -1, np.int32)
    T = np.full((m, m, m, 3), 0xFFFF, np.uint16)
    Phi = np.zeros((r, r, r, 3), np.uint8)
    Phi[g["h1"][0], g["h1"][1], 0] = g["phi_at_h1"] + [0]
    sx, sy = g["slot"]
    H[sx, sy, 0] = g["H_at_slot"][0]
    T[sx, sy, 0] = g["T_at_slot"] + [0]
    tables = [dict(m=m, r=r, H=H.reshape(-1), T=T.reshape(-1, 3), Phi=Phi.reshape(-1, 3))]
    coords = np.zeros((g["n"][0], 3), np.int32)          # only n matters here
    L = oracle.Level(coords, [0, g["n"][0]], 16, tables=tables)
    assert L.hash_slot(0, (qx, qy, 0)) == (sx * m + sy) * m + 0
    assert L.lookup(0, (qx, qy, 0)) == g["H_at_slot"][0]
    # same h0 and h1 as the query (shifted by lcm(m, r) = 6) but another pixel: tag mismatch
    assert L.hash_slot(0, (qx + 6, qy, 0)) == (sx * m + sy) * m
    assert L.lookup(0, (qx + 6, qy, 0)) == -1
    # a pixel that lands on the redundant slot: h1 = (0,0) has offset (0,0) in this table
    rx, ry = g["redundant_slot"]
    assert g["H_at_redundant"] == [-1]
    assert L.hash_slot(0, (rx, ry + 3, 0)) != (sx * m + sy) * m      # different slot
    p = (2, 4, 0)                                                     # h1=(0,0), h0=(2,1)
    assert L.hash_slot(0, p) == (rx * m + ry) * m
    assert L.lookup(0, p) == -1
    # off-grid positions are empty, never hashed
    assert L.lookup(0, (-1, 0, 0)) == -1 and L.lookup(0, (0, 16, 0)) == -1


def test_batch_offsets_second_model(oracle):
    """Fig. 3 caption: the second model's hash base is the size of the first table
    (9 = 3^2 in the 2-D figure, m^d in general) and the prefix arrays are plain
    cumulative sums with a leading zero (Section 3.2)."""
    g = _read_golden("psh_worked_example_2d.txt")
    assert g["second_model_base"][0] == g["m"][0] ** 2
    rng = np.random.default_rng(0)
    coords, offs = [], [0]
    for n in (8, 8, 30, 1):
        lin = rng.choice(16 ** 3, size=n, replace=False)
        lin.sort()
        coords.append(np.stack([lin // 256, (lin // 16) % 16, lin % 16], 1))
        offs.append(offs[-1] + n)
    L = oracle.Level(np.concatenate(coords).astype(np.int32), offs, 16)
    assert L.mbar[0] == 3 and L.M[1] == 3 ** 3
    assert np.array_equal(L.M, np.concatenate([[0], np.cumsum(L.mbar.astype(np.int64) ** 3)]))
    assert np.array_equal(L.R, np.concatenate([[0], np.cumsum(L.rbar.astype(np.int64) ** 3)]))
    assert np.array_equal(L.N, np.asarray(offs))
    assert L.H.size == L.M[-1] and L.T.shape == (L.M[-1], 3) and L.Phi.shape == (L.R[-1], 3)
    for v in range(L.b):
        assert (L.V[L.M[v]:L.M[v + 1]] == v).all()


# --------------------------------------------------------------------------------------
# size rules
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("n", [1, 2, 7, 8, 9, 26, 27, 28, 63, 64, 65, 999, 1000, 1001, 3176,
                               140607, 140608, 2_000_000])
def test_size_rules(oracle, n):
    """Section 5.2: m is the smallest side with m^3 > n; r starts at the smallest side
    with r^3 >= n/6 (then moves up to the next side coprime with m); the memory
    overhead m^3 - n obeys the bound behind Eq.9."""
    m = oracle.mbar(n)
    assert (m - 1) ** 3 <= n < m ** 3
    assert m ** 3 - n <= 3 * m * m - 3 * m + 1
    r = oracle.rbar0(n, m)
    r_plain = 1
    while 6 * r_plain ** 3 < n:
        r_plain += 1
    assert 6 * (r_plain - 1) ** 3 < n <= 6 * r_plain ** 3
    assert r >= r_plain and np.gcd(r, m) == 1
    assert all(np.gcd(k, m) != 1 for k in range(r_plain, r))
    r2 = oracle.rbar_next(r, m)
    assert r2 > r and r2 ** 3 >= 2 * r ** 3 and np.gcd(r2, m) == 1
    k = r + 1
    while k ** 3 < 2 * r ** 3 or np.gcd(k, m) != 1:
        k += 1
    assert r2 == k


def test_eight_voxels_need_a_3_table(oracle):
    # the figure's 8 occupied cells get one redundant slot in d = 2 (9 > 8); the same
    # strict rule in d = 3 gives m = 3 (27 > 8), not m = 2 (8 is not > 8)
    assert oracle.mbar(8) == 3 and oracle.mbar(7) == 2


# --------------------------------------------------------------------------------------
# validity of constructed tables
# --------------------------------------------------------------------------------------

def _check_level_valid(L, exhaustive=True):
    u = L.ubar
    for v in range(L.b):
        c = L.coords[L.N[v]:L.N[v + 1]]
        n = c.shape[0]
        m, r = int(L.mbar[v]), int(L.rbar[v])
        H = L.H[L.M[v]:L.M[v + 1]]
        T = L.T[L.M[v]:L.M[v + 1]]
        Phi = L.Phi[L.R[v]:L.R[v + 1]]
        assert (m - 1) ** 3 <= n < m ** 3 and np.gcd(m, r) == 1
        # exactly n used slots, holding a permutation of 0..n-1
        used = H != -1
        assert used.sum() == n
        assert np.array_equal(np.sort(H[used]), np.arange(n))
        # empty slots carry the empty tag, offsets stay below m
        assert (T[~used] == 0xFFFF).all()
        assert (Phi < m).all()
        # every voxel of S: its own slot, tag equal to itself, index equal to its rank
        got, slots = numpy_lookup(L, v, c)
        assert np.array_equal(got, L.N[v] + np.arange(n))
        assert np.unique(slots).size == n
        assert np.array_equal(T[slots - L.M[v]].astype(np.int32), c)
        # every voxel outside S is rejected
        if exhaustive:
            ax = np.arange(u)
            P = np.stack(np.meshgrid(ax, ax, ax, indexing="ij"), -1).reshape(-1, 3)
        else:
            P = np.random.default_rng(v).integers(0, u, size=(200000, 3))
        vol = dense_index_volume(c, u)
        truth = vol[P[:, 0], P[:, 1], P[:, 2]]
        truth = np.where(truth >= 0, truth + L.N[v], -1)
        got, _ = numpy_lookup(L, v, P)
        assert np.array_equal(got, truth)


def test_psh_valid_sphere_two_levels(oracle):
    coords, _ = S.sphere_shell_32()
    assert coords.shape[0] == 3176
    levels = oracle.build_hierarchy(coords, [0, coords.shape[0]], 32, 2)
    assert [L.ubar for L in levels] == [32, 16]
    assert levels[0].mbar[0] == 15                      # 14^3 = 2744 <= 3176 < 3375
    for L in levels:
        _check_level_valid(L)


def test_psh_valid_random_batch(oracle):
    coords, offs, _ = S.config_batch(2, batch=6)
    levels = oracle.build_hierarchy(coords, offs, 64, 3)
    for L in levels:
        _check_level_valid(L)


def test_oracle_lookup_matches_dense_volume(oracle):
    """The C lookup itself (not the numpy restatement) against the dense volume, on all
    positions of a small grid including a one-voxel rim outside it."""
    coords, offs, _ = S.config_batch(2, batch=2, u=32)
    L = oracle.Level(coords, offs, 32)
    for v in range(2):
        c = coords[offs[v]:offs[v + 1]]
        vol = dense_index_volume(c, 32)
        rng = np.random.default_rng(5 + v)
        P = rng.integers(-1, 33, size=(4000, 3))
        for p in np.concatenate([P, c[:200]]):
            inside = ((p >= 0) & (p < 32)).all()
            want = int(vol[p[0], p[1], p[2]]) if inside else -1
            want = want + int(L.N[v]) if want >= 0 else -1
            assert L.lookup(v, p) == want


def test_coarse_levels_are_parent_sets(oracle):
    coords, offs, _ = S.config_batch(2, batch=3)
    levels = oracle.build_hierarchy(coords, offs, 64, 4)
    for lf, lc in zip(levels[:-1], levels[1:]):
        assert lc.ubar * 2 == lf.ubar
        for v in range(lf.b):
            f = lf.coords[lf.N[v]:lf.N[v + 1]]
            c = lc.coords[lc.N[v]:lc.N[v + 1]]
            parents = {tuple(p) for p in (f // 2)}
            assert parents == {tuple(p) for p in c}
            lin = (c[:, 0].astype(np.int64) * lc.ubar + c[:, 1]) * lc.ubar + c[:, 2]
            assert (np.diff(lin) > 0).all()


def test_forced_failure_grows_r(oracle):
    """Two voxels congruent modulo both m and r can never be separated: the first
    attempt must fail and r must grow by the cube root of two (Section 5.2), here
    2 -> 3 -> (coprime with m = 3) 4, which separates them."""
    pts = np.array([[0, 0, 0], [6, 0, 0], [1, 2, 3], [2, 1, 1], [3, 3, 0], [4, 0, 2], [5, 5, 5],
                    [7, 7, 7]], np.int32)
    t = oracle.psh_build(pts, 32)
    assert t["m"] == 3 and t["attempts"] == 2 and t["r"] == 4
    L = oracle.Level(pts, [0, 8], 32, tables=[t])
    _check_level_valid(L)


def test_build_rejects_bad_input(oracle):
    with pytest.raises(RuntimeError):
        oracle.psh_build(np.array([[0, 0, 40]], np.int32), 32)
    with pytest.raises(RuntimeError):
        oracle.psh_build(np.array([[0, -1, 0]], np.int32), 32)


# --------------------------------------------------------------------------------------
# traversal index lists
# --------------------------------------------------------------------------------------

def test_neighbour_lists_brute_force(oracle):
    coords, offs, _ = S.config_batch(2, batch=3)
    L = oracle.Level(coords, offs, 64)
    nb = oracle.neighbours(L)
    assert nb.shape == (L.Ntot, 27) and nb.min() >= -1
    for v in range(L.b):
        c = coords[offs[v]:offs[v + 1]]
        vol = np.full((66, 66, 66), -1, np.int64)
        vol[c[:, 0] + 1, c[:, 1] + 1, c[:, 2] + 1] = np.arange(c.shape[0]) + offs[v]
        k = 0
        for dx in (-1, 0, 1):
            for dy in (-1, 0, 1):
                for dz in (-1, 0, 1):
                    want = vol[c[:, 0] + 1 + dx, c[:, 1] + 1 + dy, c[:, 2] + 1 + dz]
                    assert np.array_equal(nb[offs[v]:offs[v + 1], k], want), (v, k)
                    k += 1
    # symmetry of 3x3x3 stride-1 neighbourhoods
    i, k = np.nonzero(nb >= 0)
    assert np.array_equal(nb[nb[i, k], 26 - k], i)
    assert np.array_equal(nb[:, 13], np.arange(L.Ntot))


def test_child_lists_brute_force(oracle):
    coords, offs, _ = S.config_batch(2, batch=3)
    lf, lc = oracle.build_hierarchy(coords, offs, 64, 2)
    ch = oracle.children(lf, lc)
    assert ch.shape == (lc.Ntot, 8)
    for v in range(lf.b):
        f = lf.coords[lf.N[v]:lf.N[v + 1]]
        c = lc.coords[lc.N[v]:lc.N[v + 1]]
        vol = dense_index_volume(f, 64)
        k = 0
        for dx in (0, 1):
            for dy in (0, 1):
                for dz in (0, 1):
                    want = vol[2 * c[:, 0] + dx, 2 * c[:, 1] + dy, 2 * c[:, 2] + dz]
                    want = np.where(want >= 0, want + lf.N[v], -1)
                    assert np.array_equal(ch[lc.N[v]:lc.N[v + 1], k], want)
                    k += 1
    assert ((ch >= 0).sum(1) >= 1).all()
    # every fine voxel is the child of exactly one coarse voxel
    assert np.array_equal(np.sort(ch[ch >= 0]), np.arange(lf.Ntot))


def test_generator_is_deterministic_and_symmetric():
    c1, n1 = S.sphere_shell_32()
    c2, _ = S.sphere_shell_32()
    assert np.array_equal(c1, c2)
    s = {tuple(p) for p in c1}
    assert {(31 - x, y, z) for x, y, z in s} == s and {(y, z, x) for x, y, z in s} == s
    a = S.config_batch(2, batch=2)
    b = S.config_batch(2, batch=2)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
