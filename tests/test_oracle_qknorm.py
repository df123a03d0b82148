"""Pins for the oracle's per-head QK normalisation + 3D RoPE and its gradients (CPU only).

The paper (Section 4.5.1) only says that Q and K are normalised per head; the RMS form with a
learned gain is this build's reading, so the pins fix that reading against the mathematics:
closed forms, invariances, finite differences and an independently written PyTorch fp64
formulation (complex multiplication for the rotation, autograd for the gradients).
"""
import numpy as np
import pytest

from oracle import vfm_oracle as orc

GRIDS = [(2, 3, 4), (1, 1, 5), (3, 2, 2)]
CU = np.concatenate([[0], np.cumsum([t * h * w for t, h, w in GRIDS])])
TOTAL = int(CU[-1])
HEADS, D = 3, 16
DIMS = (4, 6, 6)
THETA = 10000.0


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_unit_gain_gives_unit_rms_rows():
    x = 3.0 * _rand((TOTAL, HEADS, D), 0) + 0.5
    y = orc.qknorm_rope3d(x, np.ones(D), 0.0, GRIDS, CU, DIMS, THETA)
    # the rotation keeps each pair's norm, so the row RMS after RoPE is still 1
    np.testing.assert_allclose(np.sqrt(np.mean(y * y, axis=2)), 1.0, rtol=0, atol=1e-13)


def test_eps_shrinks_rows_by_the_closed_form_factor():
    x = _rand((TOTAL, HEADS, D), 1)
    eps = 0.37
    y = orc.qknorm_rope3d(x, np.ones(D), eps, GRIDS, CU, DIMS, THETA)
    ms = np.mean(x * x, axis=2)
    np.testing.assert_allclose(np.mean(y * y, axis=2), ms / (ms + eps), rtol=1e-13)


def test_scale_invariance_without_eps():
    x = _rand((TOTAL, HEADS, D), 2)
    g = _rand((D,), 3)
    a = orc.qknorm_rope3d(x, g, 0.0, GRIDS, CU, DIMS, THETA)
    b = orc.qknorm_rope3d(7.25 * x, g, 0.0, GRIDS, CU, DIMS, THETA)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_unit_rms_input_reduces_to_plain_rope():
    x = _rand((TOTAL, HEADS, D), 4)
    x /= np.sqrt(np.mean(x * x, axis=2, keepdims=True))
    y = orc.qknorm_rope3d(x, np.ones(D), 0.0, GRIDS, CU, DIMS, THETA)
    np.testing.assert_allclose(y, orc.rope3d(x, GRIDS, CU, DIMS, THETA), rtol=0, atol=1e-13)


def test_origin_token_is_normalised_and_scaled_only():
    x = _rand((TOTAL, HEADS, D), 5)
    g = _rand((D,), 6)
    y = orc.qknorm_rope3d(x, g, 1e-6, GRIDS, CU, DIMS, THETA)
    for s in range(len(GRIDS)):
        n0 = int(CU[s])            # position (0,0,0) of each clip: rotation by angle 0
        want = x[n0] / np.sqrt(np.mean(x[n0] ** 2, axis=1, keepdims=True) + 1e-6) * g
        np.testing.assert_allclose(y[n0], want, rtol=0, atol=1e-14)


def test_one_hot_gain_keeps_only_that_pair():
    x = _rand((TOTAL, HEADS, D), 7)
    for d in (0, 5, D - 1):
        g = np.zeros(D)
        g[d] = 2.0
        y = orc.qknorm_rope3d(x, g, 0.0, GRIDS, CU, DIMS, THETA)
        pair = (d // 2) * 2
        mask = np.ones(D, bool)
        mask[pair:pair + 2] = False
        assert np.all(y[:, :, mask] == 0.0)
        # the rotated pair has the norm of the single scaled element
        n = x / np.sqrt(np.mean(x * x, axis=2, keepdims=True))
        np.testing.assert_allclose(np.hypot(y[:, :, pair], y[:, :, pair + 1]), np.abs(2.0 * n[:, :, d]),
                                   rtol=1e-12, atol=1e-14)


def test_gradients_match_central_differences():
    grids = [(1, 2, 2), (2, 1, 1)]
    cu = np.array([0, 4, 6])
    x = _rand((6, 2, 8), 8)
    g = 1.0 + 0.3 * _rand((8,), 9)
    dy = _rand((6, 2, 8), 10)
    eps, dims = 1e-3, (2, 2, 4)
    dx, dg = orc.qknorm_rope3d_bwd(x, g, eps, dy, grids, cu, dims, THETA)

    def loss(xx, gg):
        return float(np.sum(orc.qknorm_rope3d(xx, gg, eps, grids, cu, dims, THETA) * dy))

    h = 1e-6
    num_dx = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        num_dx[idx] = (loss(xp, g) - loss(xm, g)) / (2 * h)
    num_dg = np.zeros_like(g)
    for d in range(g.size):
        gp, gm = g.copy(), g.copy()
        gp[d] += h
        gm[d] -= h
        num_dg[d] = (loss(x, gp) - loss(x, gm)) / (2 * h)
    np.testing.assert_allclose(dx, num_dx, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dg, num_dg, rtol=1e-6, atol=1e-8)


def test_dx_is_orthogonal_to_x_without_eps():
    # scale invariance of the forward means the gradient has no component along x
    x = _rand((TOTAL, HEADS, D), 11)
    g = _rand((D,), 12)
    dy = _rand((TOTAL, HEADS, D), 13)
    dx, _ = orc.qknorm_rope3d_bwd(x, g, 0.0, dy, GRIDS, CU, DIMS, THETA)
    np.testing.assert_allclose(np.sum(dx * x, axis=2), 0.0, rtol=0, atol=1e-12)


def test_against_independent_torch_formulation():
    torch = pytest.importorskip("torch")
    x = _rand((TOTAL, HEADS, D), 14)
    g = 1.0 + 0.2 * _rand((D,), 15)
    dy = _rand((TOTAL, HEADS, D), 16)
    eps = 1e-6
    # positions by nested enumeration, angles per axis, rotation as complex multiplication
    pos = []
    for (T, H, W) in GRIDS:
        pos += [(t, h, w) for t in range(T) for h in range(H) for w in range(W)]
    pos = torch.tensor(pos, dtype=torch.float64)
    ang = []
    for axis, d_a in enumerate(DIMS):
        freq = THETA ** (-torch.arange(0, d_a, 2, dtype=torch.float64) / d_a)
        ang.append(pos[:, axis:axis + 1] * freq[None, :])
    rot = torch.polar(torch.ones(TOTAL, D // 2, dtype=torch.float64), torch.cat(ang, dim=1))
    xt = torch.tensor(x, requires_grad=True)
    gt = torch.tensor(g, requires_grad=True)
    z = xt * torch.rsqrt((xt * xt).mean(dim=-1, keepdim=True) + eps) * gt
    zc = torch.view_as_complex(z.reshape(TOTAL, HEADS, D // 2, 2))
    yt = torch.view_as_real(zc * rot[:, None, :]).reshape(TOTAL, HEADS, D)
    (yt * torch.tensor(dy)).sum().backward()
    y = orc.qknorm_rope3d(x, g, eps, GRIDS, CU, DIMS, THETA)
    dx, dg = orc.qknorm_rope3d_bwd(x, g, eps, dy, GRIDS, CU, DIMS, THETA)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), rtol=0, atol=1e-11)
