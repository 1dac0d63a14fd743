"""Pins of the CPU oracle's operators (CPU only): convolution, its two gradients and
max-pooling, against dense brute force (torch's dense float64 conv3d / max_pool3d on
zero-padded grids), closed-form special cases and adjoint identities.
"""
import numpy as np
import pytest
import torch

import synth_shapes as S


def dense_scatter(coords, X, u, fill=0.0):
    """voxel-major rows X [n,c] -> dense [c,u,u,u] float64."""
    c = X.shape[1]
    vol = np.full((c, u, u, u), fill, np.float64)
    vol[:, coords[:, 0], coords[:, 1], coords[:, 2]] = X.T
    return vol


def dense_conv_masked(coords, offs, X, W, u):
    """Zero-padded dense 3-D cross-correlation per model, read back at the occupied
    voxels.  W is [27, c_in, c_out], tap k = (dx+1)*9 + (dy+1)*3 + (dz+1)."""
    c_in, c_out = W.shape[1], W.shape[2]
    wt = torch.from_numpy(np.asarray(W, np.float64).reshape(3, 3, 3, c_in, c_out)
                          .transpose(4, 3, 0, 1, 2).copy())
    out = np.empty((X.shape[0], c_out), np.float64)
    for v in range(len(offs) - 1):
        c = coords[offs[v]:offs[v + 1]]
        vol = torch.from_numpy(dense_scatter(c, np.asarray(X[offs[v]:offs[v + 1]], np.float64), u))
        y = torch.nn.functional.conv3d(vol[None], wt, padding=1)[0].numpy()
        out[offs[v]:offs[v + 1]] = y[:, c[:, 0], c[:, 1], c[:, 2]].T
    return out


@pytest.fixture(scope="module")
def small_batch(oracle):
    coords, offs, normals = S.config_batch(2, batch=3, u=32, with_normals=True)
    L = oracle.Level(coords, offs, 32)
    return coords, offs, normals, L


def test_conv_fwd_config1_vs_dense(oracle):
    """The single-sphere case: 3 -> 16 channels, weights N(0, 0.1) seed 0."""
    coords, normals = S.sphere_shell_32()
    L = oracle.Level(coords, [0, coords.shape[0]], 32)
    W = S.gaussian((27, 3, 16), 0.1, 0)
    Y = oracle.from_paper_X(oracle.conv_fwd(L, oracle.to_paper_X(normals), oracle.to_paper_W(W)))
    want = dense_conv_masked(coords, [0, coords.shape[0]], normals, W, 32)
    np.testing.assert_allclose(Y, want, rtol=0, atol=1e-12)


def test_conv_fwd_batch_vs_dense(oracle, small_batch):
    coords, offs, normals, L = small_batch
    X = S.normals_plus_one(normals)
    W = S.gaussian((27, 4, 5), 0.05, 1)
    Y = oracle.from_paper_X(oracle.conv_fwd(L, oracle.to_paper_X(X), oracle.to_paper_W(W)))
    want = dense_conv_masked(coords, offs, X, W, 32)
    np.testing.assert_allclose(Y, want, rtol=0, atol=1e-12)
    # Eq.2 evaluated voxel by voxel agrees with the matrix form Eq.3
    idx = np.random.default_rng(0).choice(L.Ntot, 300, replace=False)
    Ys = oracle.conv_fwd_at(L, oracle.to_paper_X(X), oracle.to_paper_W(W), idx)
    np.testing.assert_allclose(Ys, want[idx], rtol=0, atol=1e-12)


def test_hash2col_is_a_gather_of_neighbours(oracle, small_batch):
    coords, offs, normals, L = small_batch
    X = S.gaussian((L.Ntot, 3), 1.0, 2).astype(np.float64)
    Dt = oracle.hash2col(L, L, oracle.to_paper_X(X))                 # (3*27) x N
    vol = [np.pad(dense_scatter(coords[offs[v]:offs[v + 1]], X[offs[v]:offs[v + 1]], 32),
                  ((0, 0), (1, 1), (1, 1), (1, 1))) for v in range(L.b)]
    for v in range(L.b):
        c = coords[offs[v]:offs[v + 1]]
        k = 0
        for dx in (-1, 0, 1):
            for dy in (-1, 0, 1):
                for dz in (-1, 0, 1):
                    want = vol[v][:, c[:, 0] + 1 + dx, c[:, 1] + 1 + dy, c[:, 2] + 1 + dz]
                    for ic in range(3):
                        assert np.array_equal(Dt[ic * 27 + k, offs[v]:offs[v + 1]], want[ic])
                    k += 1


def test_conv_special_cases(oracle, small_batch):
    coords, offs, normals, L = small_batch
    rng = np.random.default_rng(3)
    # centre tap only: a plain per-voxel matrix product
    X = rng.standard_normal((L.Ntot, 4))
    W = np.zeros((27, 4, 6))
    W[13] = rng.standard_normal((4, 6))
    Y = oracle.from_paper_X(oracle.conv_fwd(L, oracle.to_paper_X(X), oracle.to_paper_W(W)))
    np.testing.assert_allclose(Y, X @ W[13], rtol=0, atol=1e-13)
    # all-ones: the output counts the occupied neighbours
    ones = np.ones((L.Ntot, 1))
    Y = oracle.from_paper_X(oracle.conv_fwd(L, oracle.to_paper_X(ones),
                                            oracle.to_paper_W(np.ones((27, 1, 1)))))
    nb = oracle.neighbours(L)
    assert np.array_equal(Y[:, 0], (nb >= 0).sum(1).astype(np.float64))
    # one off-centre tap picks exactly that neighbour (orientation of k)
    W = np.zeros((27, 1, 1))
    k = 2 * 9 + 0 * 3 + 1            # delta = (+1, -1, 0)
    W[k] = 1.0
    x = rng.standard_normal((L.Ntot, 1))
    Y = oracle.from_paper_X(oracle.conv_fwd(L, oracle.to_paper_X(x), oracle.to_paper_W(W)))
    for v in range(L.b):
        c = coords[offs[v]:offs[v + 1]]
        vol = np.pad(dense_scatter(c, x[offs[v]:offs[v + 1]], 32), ((0, 0), (1, 1), (1, 1), (1, 1)))
        want = vol[0, c[:, 0] + 2, c[:, 1] + 0, c[:, 2] + 1]
        assert np.array_equal(Y[offs[v]:offs[v + 1], 0], want)


def test_config1_axis_permutation_equivariance(oracle):
    """The sphere and its normals are symmetric under axis permutation: permuting the
    axes of the input, of the weights' taps and of the normal components permutes the
    output the same way."""
    coords, normals = S.sphere_shell_32()
    L = oracle.Level(coords, [0, coords.shape[0]], 32)
    W = S.gaussian((27, 3, 4), 0.1, 7).astype(np.float64)
    Y = oracle.from_paper_X(oracle.conv_fwd(L, oracle.to_paper_X(normals), oracle.to_paper_W(W)))
    perm = [1, 2, 0]
    # voxel (x,y,z) -> (y,z,x): find the index of each permuted voxel
    lut = {tuple(p): i for i, p in enumerate(coords)}
    j = np.array([lut[tuple(p[perm])] for p in coords])
    Wp = W.reshape(3, 3, 3, 3, 4).transpose(*perm, 3, 4)[:, :, :, perm, :].reshape(27, 3, 4)
    # the normal at the permuted voxel is the permuted normal: the input maps to itself
    np.testing.assert_allclose(normals[j], normals[:, perm], atol=1e-6)
    Y2 = oracle.from_paper_X(oracle.conv_fwd(L, oracle.to_paper_X(normals),
                                             oracle.to_paper_W(Wp)))
    np.testing.assert_allclose(Y2[j], Y, rtol=0, atol=1e-6)


def test_gradients_vs_dense_autograd(oracle, small_batch):
    """Eq.7 and Eq.8 + col2hash against torch autograd through the dense masked conv."""
    coords, offs, normals, L = small_batch
    rng = np.random.default_rng(4)
    c_in, c_out, u = 3, 4, 32
    X = rng.standard_normal((L.Ntot, c_in))
    W = rng.standard_normal((27, c_in, c_out)) * 0.1
    G = rng.standard_normal((L.Ntot, c_out))
    wt = torch.from_numpy(W.reshape(3, 3, 3, c_in, c_out).transpose(4, 3, 0, 1, 2).copy())
    wt.requires_grad_(True)
    dX_want = np.empty_like(X)
    for v in range(L.b):
        c = torch.from_numpy(coords[offs[v]:offs[v + 1]].astype(np.int64))
        xv = torch.from_numpy(X[offs[v]:offs[v + 1]].copy()).requires_grad_(True)
        lin = (c[:, 0] * u + c[:, 1]) * u + c[:, 2]
        vol = torch.zeros((u * u * u, c_in), dtype=torch.float64).index_put((lin,), xv)
        vol = vol.T.reshape(c_in, u, u, u)
        y = torch.nn.functional.conv3d(vol[None], wt, padding=1)[0]
        ys = y[:, c[:, 0], c[:, 1], c[:, 2]].T
        (ys * torch.from_numpy(G[offs[v]:offs[v + 1]])).sum().backward()
        dX_want[offs[v]:offs[v + 1]] = xv.grad.numpy()
    dW_want = wt.grad.numpy().transpose(2, 3, 4, 1, 0).reshape(27, c_in, c_out)
    Wp = oracle.to_paper_W(W)
    dX = oracle.from_paper_X(oracle.conv_bwd_data(L, oracle.to_paper_X(G), Wp, c_in))
    dW = oracle.from_paper_W(oracle.conv_bwd_weight(L, oracle.to_paper_X(X), oracle.to_paper_X(G)),
                             c_in)
    np.testing.assert_allclose(dX, dX_want, rtol=0, atol=1e-11)
    np.testing.assert_allclose(dW, dW_want, rtol=0, atol=1e-10)
    # sampled forms agree
    idx = rng.choice(L.Ntot, 200, replace=False)
    np.testing.assert_allclose(oracle.conv_bwd_data_at(L, oracle.to_paper_X(G), Wp, c_in, idx),
                               dX_want[idx], rtol=0, atol=1e-11)
    tr = np.stack([rng.integers(0, c_out, 40), rng.integers(0, c_in, 40),
                   rng.integers(0, 27, 40)], 1)
    got = oracle.conv_bwd_weight_at(L, oracle.to_paper_X(X), oracle.to_paper_X(G), tr)
    np.testing.assert_allclose(got, dW_want[tr[:, 2], tr[:, 1], tr[:, 0]], rtol=0, atol=1e-10)


def test_adjoint_identities(oracle, small_batch):
    """<conv(X;W), G> = <X, bwd_data(G;W)> = <W, bwd_weight(X,G)>, and col2hash is the
    transpose of hash2col."""
    coords, offs, normals, L = small_batch
    rng = np.random.default_rng(5)
    c_in, c_out = 5, 3
    X = rng.standard_normal((c_in, L.Ntot))
    Wp = rng.standard_normal((c_out, c_in * 27))
    G = rng.standard_normal((c_out, L.Ntot))
    lhs = (oracle.conv_fwd(L, X, Wp) * G).sum()
    assert abs(lhs - (X * oracle.conv_bwd_data(L, G, Wp, c_in)).sum()) < 1e-9 * abs(lhs)
    assert abs(lhs - (Wp * oracle.conv_bwd_weight(L, X, G)).sum()) < 1e-9 * abs(lhs)
    Cm = rng.standard_normal((c_in * 27, L.Ntot))
    a = (oracle.hash2col(L, L, X) * Cm).sum()
    b = (X * oracle.col2hash(L, L, Cm, c_in)).sum()
    assert abs(a - b) < 1e-9 * abs(a)
    # col2hash(hash2col(1)) counts the occupied neighbours
    ones = np.ones((1, L.Ntot))
    cnt = oracle.col2hash(L, L, oracle.hash2col(L, L, ones), 1)
    assert np.array_equal(cnt[0], (oracle.neighbours(L) >= 0).sum(1).astype(np.float64))


def test_matmul_vs_numpy(oracle):
    rng = np.random.default_rng(6)
    A, B = rng.standard_normal((7, 11)), rng.standard_normal((11, 5))
    np.testing.assert_allclose(oracle.matmul(A, B), A @ B, atol=1e-13)
    np.testing.assert_allclose(oracle.matmul(A.T.copy(), B, ta=True), A @ B, atol=1e-13)
    np.testing.assert_allclose(oracle.matmul(A, B.T.copy(), tb=True), A @ B, atol=1e-13)
    np.testing.assert_allclose(oracle.matmul(A.T.copy(), B.T.copy(), ta=True, tb=True), A @ B,
                               atol=1e-13)


def test_max_pool_vs_dense(oracle):
    """Dense 2x2x2 max-pool with -inf at empty voxels; the switch must be an occupied
    child of the right parent holding the maximum; ties go to the first child."""
    coords, offs, _ = S.config_batch(2, batch=3)
    lf, lc = oracle.build_hierarchy(coords, offs, 64, 2)
    rng = np.random.default_rng(8)
    c = 5
    X = rng.standard_normal((lf.Ntot, c))
    X[rng.random(X.shape) < 0.5] = 0.0            # many ties at zero, as after ReLU
    Y, sw = oracle.pool_max_fwd(lf, lc, oracle.to_paper_X(X))
    Y, sw = Y.T, sw.T
    ch = oracle.children(lf, lc)
    for v in range(lf.b):
        f = lf.coords[lf.N[v]:lf.N[v + 1]]
        cc = lc.coords[lc.N[v]:lc.N[v + 1]]
        vol = torch.from_numpy(dense_scatter(f, X[lf.N[v]:lf.N[v + 1]], 64, fill=-np.inf))
        want = torch.nn.functional.max_pool3d(vol[None], 2)[0].numpy()
        np.testing.assert_array_equal(Y[lc.N[v]:lc.N[v + 1]],
                                      want[:, cc[:, 0], cc[:, 1], cc[:, 2]].T)
    # switches: an occupied child of the same parent, value equal to the max, and the
    # first such child in k order
    for ic in range(c):
        vals = np.where(ch >= 0, X[np.maximum(ch, 0), ic], -np.inf)
        first = vals.argmax(1)                    # numpy argmax returns the first maximum
        assert np.array_equal(sw[:, ic], ch[np.arange(lc.Ntot), first])
    # backward: only the switches receive gradient, sums are preserved (fields disjoint)
    dY = rng.standard_normal((lc.Ntot, c))
    dX = oracle.pool_max_bwd(lf.Ntot, oracle.to_paper_X(dY), sw.T.copy()).T
    np.testing.assert_allclose(dX.sum(0), dY.sum(0), atol=1e-9)
    mask = np.zeros_like(dX, bool)
    for ic in range(c):
        mask[sw[:, ic], ic] = True
        assert np.array_equal(dX[sw[:, ic], ic], dY[:, ic])
    assert (dX[~mask] == 0).all()


def test_strided_traversal_general_form(oracle):
    """Algorithm 1's strided receptive field [p*Ss - Sp, p*Ss - Sp + F - 1]^3 with F = 3,
    Ss = 2, Sp = 1 across two levels, against the dense index volume."""
    coords, offs, _ = S.config_batch(2, batch=2)
    lf, lc = oracle.build_hierarchy(coords, offs, 64, 2)
    fi = oracle.field_indices(lf, lc, F=3, Ss=2, Sp=1)
    for v in range(lf.b):
        f = lf.coords[lf.N[v]:lf.N[v + 1]]
        cc = lc.coords[lc.N[v]:lc.N[v + 1]].astype(np.int64)
        vol = np.full((66, 66, 66), -1, np.int64)
        vol[f[:, 0] + 1, f[:, 1] + 1, f[:, 2] + 1] = np.arange(f.shape[0]) + lf.N[v]
        row = 0
        for fx in range(3):
            for fy in range(3):
                for fz in range(3):
                    want = vol[2 * cc[:, 0] - 1 + fx + 1, 2 * cc[:, 1] - 1 + fy + 1,
                               2 * cc[:, 2] - 1 + fz + 1]
                    assert np.array_equal(fi[lc.N[v]:lc.N[v + 1], row], want)
                    row += 1


def test_deconv_vs_dense_conv_transpose(oracle, small_batch):
    """Transposed convolution against torch's dense float64 conv_transpose3d read back at the
    occupied voxels, and as the adjoint of the forward convolution."""
    coords, offs, normals, L = small_batch
    rng = np.random.default_rng(11)
    c_i, c_o, u = 4, 3, 32
    X = rng.standard_normal((L.Ntot, c_i))
    W = rng.standard_normal((27, c_o, c_i)) * 0.1        # forward conv c_o -> c_i
    wt = torch.from_numpy(W.reshape(3, 3, 3, c_o, c_i).transpose(4, 3, 0, 1, 2).copy())   # [c_i, c_o, 3,3,3]
    want = np.empty((L.Ntot, c_o))
    for v in range(L.b):
        c = coords[offs[v]:offs[v + 1]]
        vol = torch.from_numpy(dense_scatter(c, X[offs[v]:offs[v + 1]], u))
        # conv_transpose3d's weight is [in, out, k...] and it is the adjoint of conv3d with the
        # same tensor read as [out_fwd = in, in_fwd = out]
        y = torch.nn.functional.conv_transpose3d(vol[None], wt, padding=1)[0].numpy()
        want[offs[v]:offs[v + 1]] = y[:, c[:, 0], c[:, 1], c[:, 2]].T
    Wp = oracle.to_paper_W(W)                              # c_i x (c_o*27)
    got = oracle.deconv_fwd(L, oracle.to_paper_X(X), Wp).T
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-11)
    # adjoint of the forward convolution with the same weights
    Z = rng.standard_normal((c_o, L.Ntot))
    lhs = (oracle.conv_fwd(L, Z, Wp) * oracle.to_paper_X(X)).sum()
    rhs = (Z * oracle.deconv_fwd(L, oracle.to_paper_X(X), Wp)).sum()
    assert abs(lhs - rhs) < 1e-9 * abs(lhs)


def test_unpool_restores_only_switches(oracle):
    coords, offs, _ = S.config_batch(2, batch=2)
    lf, lc = oracle.build_hierarchy(coords, offs, 64, 2)
    rng = np.random.default_rng(12)
    c = 3
    X = rng.standard_normal((c, lf.Ntot))
    P, sw = oracle.pool_max_fwd(lf, lc, X)
    U = oracle.unpool_max_fwd(lf.Ntot, P, sw)
    # unpool(pool(X)) keeps exactly the maxima: equal to X at the switches, zero elsewhere
    mask = np.zeros_like(X, bool)
    for ic in range(c):
        mask[ic, sw[ic]] = True
    assert np.array_equal(U[mask], X[mask]) and (U[~mask] == 0).all()
    # backward of unpooling is the adjoint gather
    G = rng.standard_normal((c, lf.Ntot))
    dP = oracle.unpool_max_bwd(G, sw)
    assert abs((U * G).sum() - (P * dP).sum()) < 1e-9


# --------------------------------------------------------------------------------------
# general kernel side / stride / padding across two levels, average pooling
# --------------------------------------------------------------------------------------

def _two_levels(oracle, u=32, batch=3, n_levels=2):
    coords, offs, _ = S.config_batch(2, batch=batch, u=u)
    return coords, offs, oracle.build_hierarchy(coords, offs, u, n_levels)


def _dense_strided(Li, Lo, X, W, F, Ss, Sp, u, need_grad=False):
    """dense zero-padded conv3d per model with torch (float64), read at the occupied output
    voxels; returns the outputs and, for gradients, the torch tensors."""
    c_in, c_out = W.shape[1], W.shape[2]
    wt = torch.from_numpy(np.asarray(W, np.float64).reshape(F, F, F, c_in, c_out).transpose(4, 3, 0, 1, 2).copy())
    wt.requires_grad_(need_grad)
    pad = (F - 1) // 2 if Ss == 1 else Sp
    outs, vols = [], []
    for v in range(Li.b):
        ci = Li.coords[Li.N[v]:Li.N[v + 1]]
        co = Lo.coords[Lo.N[v]:Lo.N[v + 1]]
        vol = torch.from_numpy(dense_scatter(ci, np.asarray(X[Li.N[v]:Li.N[v + 1]], np.float64), u))
        vol.requires_grad_(need_grad)
        y = torch.nn.functional.conv3d(vol[None], wt, stride=Ss, padding=pad)[0]
        outs.append(y[:, co[:, 0], co[:, 1], co[:, 2]].T)
        vols.append((vol, ci))
    return torch.cat(outs, 0), wt, vols


@pytest.mark.parametrize("F,Ss,Sp", [(3, 2, 1), (2, 2, 0), (5, 1, 2), (4, 2, 1), (3, 4, 1)])
def test_general_conv_vs_dense(oracle, F, Ss, Sp):
    """Forward and both gradients of the general traversal against dense strided conv3d and its
    autograd, outputs taken at the occupied voxels of the output level."""
    shift = {1: 0, 2: 1, 4: 2}[Ss]
    coords, offs, lv = _two_levels(oracle, n_levels=shift + 1)
    Li, Lo = lv[0], lv[shift]
    c_in, c_out = 3, 4
    X = S.gaussian((Li.Ntot, c_in), 1.0, 81)
    W = S.gaussian((F ** 3, c_in, c_out), 0.2, 82)
    G = S.gaussian((Lo.Ntot, c_out), 1.0, 83)
    Wp = oracle.to_paper_W(W)
    Y = oracle.sconv_fwd(Li, Lo, oracle.to_paper_X(X), Wp, F, Ss, Sp).T
    want, wt, vols = _dense_strided(Li, Lo, X, W, F, Ss, Sp, 32, need_grad=True)
    np.testing.assert_allclose(Y, want.detach().numpy(), rtol=0, atol=1e-11)
    (want * torch.from_numpy(G)).sum().backward()
    dW = oracle.sconv_bwd_weight(Li, Lo, oracle.to_paper_X(X), oracle.to_paper_X(G), F, Ss, Sp)
    want_dW = wt.grad.numpy().transpose(2, 3, 4, 1, 0).reshape(F ** 3, c_in, c_out)     # [row][ci][co]
    np.testing.assert_allclose(dW.reshape(c_out, c_in, F ** 3).transpose(2, 1, 0), want_dW, rtol=0, atol=1e-10)
    dX = oracle.sconv_bwd_data(Li, Lo, oracle.to_paper_X(G), Wp, c_in, F, Ss, Sp).T
    want_dX = np.concatenate([vol.grad.numpy()[:, ci[:, 0], ci[:, 1], ci[:, 2]].T for vol, ci in vols], 0)
    np.testing.assert_allclose(dX, want_dX, rtol=0, atol=1e-11)


def test_general_field_special_cases(oracle):
    """F = 3, stride 1 is the neighbour list; F = 2, stride 2, no padding the child list; the
    field of a stride-2 3^3 kernel contains the child list at its rows with all f >= 1."""
    coords, offs, lv = _two_levels(oracle)
    Li, Lo = lv[0], lv[1]
    assert np.array_equal(oracle.field_indices(Li, Li, 3, 1, 0), oracle.neighbours(Li))
    f3 = oracle.field_indices(Li, Lo, 3, 2, 1)
    rows = [((fx * 3) + fy) * 3 + fz for fx in (1, 2) for fy in (1, 2) for fz in (1, 2)]
    assert np.array_equal(f3[:, rows], oracle.children(Li, Lo))


def test_avgpool_vs_dense(oracle):
    """Average pooling = mean over the 2^3 field with empty voxels counted as zero (dense
    avg_pool3d of the zero-filled grid), and its adjoint."""
    coords, offs, lv = _two_levels(oracle)
    Li, Lo = lv[0], lv[1]
    c = 3
    X = S.gaussian((Li.Ntot, c), 1.0, 91)
    G = S.gaussian((Lo.Ntot, c), 1.0, 92)
    Y = oracle.avgpool_fwd(Li, Lo, oracle.to_paper_X(X)).T
    dX = oracle.avgpool_bwd(Li, Lo, oracle.to_paper_X(G)).T
    for v in range(Li.b):
        ci = Li.coords[Li.N[v]:Li.N[v + 1]]
        co = Lo.coords[Lo.N[v]:Lo.N[v + 1]]
        vol = torch.from_numpy(dense_scatter(ci, X[Li.N[v]:Li.N[v + 1]].astype(np.float64), 32))
        y = torch.nn.functional.avg_pool3d(vol[None], 2)[0].numpy()
        np.testing.assert_allclose(Y[Lo.N[v]:Lo.N[v + 1]], y[:, co[:, 0], co[:, 1], co[:, 2]].T, rtol=0, atol=1e-13)
        # adjoint: every fine voxel receives an eighth of its parent's value
        parent = {tuple(p): i for i, p in enumerate(co)}
        want = np.stack([G[Lo.N[v] + parent[tuple(p // 2)]] / 8.0 for p in ci])
        np.testing.assert_allclose(dX[Li.N[v]:Li.N[v + 1]], want, rtol=0, atol=1e-13)
    # <avgpool(X), G> = <X, avgpool_bwd(G)>
    assert abs((Y * G).sum() - (X * dX).sum()) < 1e-9


# --------------------------------------------------------------------------------------
# levels in ratios other than 2 (Section 4: a PSH on a grid of any resolution allows any stride)
# --------------------------------------------------------------------------------------

@pytest.mark.parametrize("u,ratio", [(30, 3), (32, 3), (35, 5)])
def test_ratio_levels_occupancy_and_max_pool(oracle, u, ratio):
    """The coarse level of ratio r is the dense occupancy max-pooled with window r (ceil mode for
    a side that r does not divide); max-pooling with F = S = r equals dense max_pool3d with
    -inf at the empty voxels, the switches point at an occupied voxel below the right parent,
    and the backward pass moves each gradient to its switch."""
    coords, offs, _ = S.config_batch(2, batch=2, u=u)
    lv = oracle.build_hierarchy(coords, offs, u, 2, ratios=[ratio])
    Li, Lo = lv[0], lv[1]
    uc = -(-u // ratio)
    assert Lo.ubar == uc
    c = 3
    X = S.gaussian((Li.Ntot, c), 1.0, 131)
    P, sw = oracle.pool_max_fwd(Li, Lo, oracle.to_paper_X(X), ratio, ratio, 0)
    for v in range(Li.b):
        ci = Li.coords[Li.N[v]:Li.N[v + 1]]
        co = Lo.coords[Lo.N[v]:Lo.N[v + 1]]
        occ = torch.zeros((1, u, u, u), dtype=torch.float64)
        occ[0, ci[:, 0], ci[:, 1], ci[:, 2]] = 1.0
        pooled = torch.nn.functional.max_pool3d(occ, ratio, ceil_mode=True)[0].numpy()
        want_c = np.argwhere(pooled > 0)
        assert np.array_equal(co, want_c)           # argwhere is in linear-index order too
        vol = torch.full((c, u, u, u), -np.inf, dtype=torch.float64)
        vol[:, ci[:, 0], ci[:, 1], ci[:, 2]] = torch.from_numpy(X[Li.N[v]:Li.N[v + 1]].astype(np.float64).T)
        want = torch.nn.functional.max_pool3d(vol[None], ratio, ceil_mode=True)[0].numpy()
        np.testing.assert_array_equal(P[:, Lo.N[v]:Lo.N[v + 1]], want[:, co[:, 0], co[:, 1], co[:, 2]])
        s = sw[:, Lo.N[v]:Lo.N[v + 1]]
        assert (s >= Li.N[v]).all() and (s < Li.N[v + 1]).all()
        assert np.array_equal(Li.coords[s] // ratio, np.broadcast_to(co, (c,) + co.shape))
    G = S.gaussian((Lo.Ntot, c), 1.0, 132)
    dX = oracle.pool_max_bwd(Li.Ntot, oracle.to_paper_X(G), sw)
    assert abs(dX.sum() - G.astype(np.float64).sum()) < 1e-9 and (dX != 0).sum() == G.size
    assert np.array_equal(dX[np.arange(c)[:, None], sw], oracle.to_paper_X(G))


@pytest.mark.parametrize("u,F,Ss,Sp", [(30, 3, 3, 0), (32, 5, 3, 1), (35, 5, 5, 0)])
def test_ratio_levels_conv_vs_dense(oracle, u, F, Ss, Sp):
    """Strided convolution and its gradients between levels in ratio 3 and 5 against dense
    conv3d with that stride (a side the stride does not divide is zero-padded at the far end,
    which is what an out-of-grid lookup returns), and average pooling against avg_pool3d."""
    coords, offs, _ = S.config_batch(2, batch=2, u=u)
    lv = oracle.build_hierarchy(coords, offs, u, 2, ratios=[Ss])
    Li, Lo = lv[0], lv[1]
    c_in, c_out = 2, 3
    X = S.gaussian((Li.Ntot, c_in), 1.0, 141)
    W = S.gaussian((F ** 3, c_in, c_out), 0.2, 142)
    G = S.gaussian((Lo.Ntot, c_out), 1.0, 143)
    Wp = oracle.to_paper_W(W)
    up = Lo.ubar * Ss + F                   # padded side: every field of every output voxel inside
    wt = torch.from_numpy(np.asarray(W, np.float64).reshape(F, F, F, c_in, c_out).transpose(4, 3, 0, 1, 2).copy())
    wt.requires_grad_(True)
    outs, vols = [], []
    for v in range(Li.b):
        ci = Li.coords[Li.N[v]:Li.N[v + 1]]
        co = Lo.coords[Lo.N[v]:Lo.N[v + 1]]
        vol = torch.zeros((c_in, up, up, up), dtype=torch.float64)
        vol[:, ci[:, 0] + Sp, ci[:, 1] + Sp, ci[:, 2] + Sp] = torch.from_numpy(X[Li.N[v]:Li.N[v + 1]].astype(np.float64).T)
        vol.requires_grad_(True)
        y = torch.nn.functional.conv3d(vol[None], wt, stride=Ss)[0]
        outs.append(y[:, co[:, 0], co[:, 1], co[:, 2]].T)
        vols.append((vol, ci))
    want = torch.cat(outs, 0)
    Y = oracle.sconv_fwd(Li, Lo, oracle.to_paper_X(X), Wp, F, Ss, Sp).T
    np.testing.assert_allclose(Y, want.detach().numpy(), rtol=0, atol=1e-11)
    (want * torch.from_numpy(G)).sum().backward()
    dW = oracle.sconv_bwd_weight(Li, Lo, oracle.to_paper_X(X), oracle.to_paper_X(G), F, Ss, Sp)
    want_dW = wt.grad.numpy().transpose(2, 3, 4, 1, 0).reshape(F ** 3, c_in, c_out)
    np.testing.assert_allclose(dW.reshape(c_out, c_in, F ** 3).transpose(2, 1, 0), want_dW, rtol=0, atol=1e-10)
    dX = oracle.sconv_bwd_data(Li, Lo, oracle.to_paper_X(G), Wp, c_in, F, Ss, Sp).T
    want_dX = np.concatenate([vol.grad.numpy()[:, ci[:, 0] + Sp, ci[:, 1] + Sp, ci[:, 2] + Sp].T for vol, ci in vols], 0)
    np.testing.assert_allclose(dX, want_dX, rtol=0, atol=1e-11)
    if F == Ss and Sp == 0:
        A = oracle.avgpool_fwd(Li, Lo, oracle.to_paper_X(X), F, Ss, Sp).T
        for v in range(Li.b):
            vol, ci = vols[v]
            co = Lo.coords[Lo.N[v]:Lo.N[v + 1]]
            a = torch.nn.functional.avg_pool3d(vol.detach()[None], F)[0].numpy()
            np.testing.assert_allclose(A[Lo.N[v]:Lo.N[v + 1]], a[:, co[:, 0], co[:, 1], co[:, 2]].T, rtol=0, atol=1e-13)
        dA = oracle.avgpool_bwd(Li, Lo, oracle.to_paper_X(G[:, :c_in]), F, Ss, Sp).T
        assert abs((A * G[:, :c_in]).sum() - (X * dA).sum()) < 1e-9
