"""Pins for the oracle's 3D RoPE and token -> (t,h,w) map (CPU only)."""
import os

import numpy as np
import pytest

from oracle import vfm_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


GRIDS = [(2, 4, 4), (3, 2, 5), (1, 1, 7)]
CU = np.concatenate([[0], np.cumsum([t * h * w for t, h, w in GRIDS])])
DIMS = (4, 6, 6)


def test_token_coords_nested_loops():
    # independent construction: enumerate the grid with t outermost, w innermost
    want = []
    for (T, H, W) in GRIDS:
        for t in range(T):
            for h in range(H):
                for w in range(W):
                    want.append((t, h, w))
    got = orc.token_coords(GRIDS, CU)
    assert got.tolist() == [list(p) for p in want]


def test_token_coords_spatial_view_is_free():
    # Section 4.6: spatial attention views [h*w*t] as [t, h*w]; with t slowest,
    # every H*W-long slice of a clip shares one t.
    pos = orc.token_coords([(3, 2, 5)], [0, 30])
    assert all(len(set(pos[f * 10:(f + 1) * 10, 0])) == 1 for f in range(3))


def test_golden_closed_form():
    rows = {}
    with open(os.path.join(GOLDEN, "rope3d_closed_form.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            rows[key] = [float(v) for v in vals]
    tok = int(rows["token"][0])
    x = np.zeros((2 * 3 * 51, 1, 8))
    x[tok, 0] = rows["x"]
    y = orc.rope3d(x, [(2, 3, 51)], [0, 306], (2, 2, 4), theta=10000.0)
    np.testing.assert_allclose(y[tok, 0], rows["y"], rtol=0, atol=1e-14)


def test_norm_preserved_per_pair():
    x = _rand((CU[-1], 3, 16), 1)
    y = orc.rope3d(x, GRIDS, CU, DIMS)
    n_in = x[..., 0::2] ** 2 + x[..., 1::2] ** 2
    n_out = y[..., 0::2] ** 2 + y[..., 1::2] ** 2
    np.testing.assert_allclose(n_out, n_in, rtol=1e-13)
    assert not np.allclose(x, y)


def test_origin_is_identity():
    x = _rand((CU[-1], 2, 16), 2)
    y = orc.rope3d(x, GRIDS, CU, DIMS)
    for a in CU[:-1]:
        np.testing.assert_array_equal(y[a], x[a])


def test_inverse_undoes_forward():
    x = _rand((CU[-1], 2, 16), 3)
    y = orc.rope3d(orc.rope3d(x, GRIDS, CU, DIMS), GRIDS, CU, DIMS, inverse=True)
    np.testing.assert_allclose(y, x, atol=1e-14)


def test_inverse_is_transpose():
    # <R x, y> == <x, R^T y>
    x = _rand((CU[-1], 2, 16), 4)
    y = _rand((CU[-1], 2, 16), 5)
    lhs = (orc.rope3d(x, GRIDS, CU, DIMS) * y).sum()
    rhs = (x * orc.rope3d(y, GRIDS, CU, DIMS, inverse=True)).sum()
    assert abs(lhs - rhs) < 1e-10


@pytest.mark.parametrize("shift", [(5, 0, 0), (0, 7, 0), (0, 0, 11), (3, 2, 9)])
def test_scores_depend_on_offsets_only(shift):
    grid, cu = [(3, 4, 5)], [0, 60]
    q = _rand((60, 2, 16), 6)
    k = _rand((60, 2, 16), 7)
    s0 = np.einsum("ihd,jhd->hij", orc.rope3d(q, grid, cu, DIMS), orc.rope3d(k, grid, cu, DIMS))
    s1 = np.einsum("ihd,jhd->hij", orc.rope3d(q, grid, cu, DIMS, pos_offset=shift),
                   orc.rope3d(k, grid, cu, DIMS, pos_offset=shift))
    np.testing.assert_allclose(s1, s0, atol=1e-11)


def test_axes_use_their_own_positions():
    # two tokens that differ only in w must agree on the t and h slices
    grid, cu = [(2, 3, 4)], [0, 24]
    x = np.tile(_rand((1, 1, 16), 8), (24, 1, 1))
    y = orc.rope3d(x, grid, cu, DIMS)
    a, b = (1 * 3 + 2) * 4 + 0, (1 * 3 + 2) * 4 + 3           # (1,2,0) and (1,2,3)
    np.testing.assert_allclose(y[a, 0, :10], y[b, 0, :10], atol=1e-15)
    assert not np.allclose(y[a, 0, 10:], y[b, 0, 10:])
    c = (0 * 3 + 2) * 4 + 0                                    # (0,2,0): differs in t only
    assert not np.allclose(y[a, 0, :4], y[c, 0, :4])
    np.testing.assert_allclose(y[a, 0, 4:], y[c, 0, 4:], atol=1e-15)


def test_reduces_to_textbook_1d_rope_complex():
    # split (D,0,0) on a (T,1,1) grid is ordinary 1-D RoPE; check the scores with
    # complex arithmetic: <R_m q, R_n k> = Re sum_i q_i conj(k_i) e^{i (m-n) theta_i}
    T, D, theta = 9, 8, 10000.0
    q = _rand((T, 1, D), 9)
    k = _rand((T, 1, D), 10)
    rq = orc.rope3d(q, [(T, 1, 1)], [0, T], (D, 0, 0), theta)
    rk = orc.rope3d(k, [(T, 1, 1)], [0, T], (D, 0, 0), theta)
    got = np.einsum("id,jd->ij", rq[:, 0], rk[:, 0])
    qc = q[:, 0, 0::2] + 1j * q[:, 0, 1::2]
    kc = k[:, 0, 0::2] + 1j * k[:, 0, 1::2]
    th = np.array([theta ** (-(2 * i) / D) for i in range(D // 2)])
    want = np.zeros((T, T))
    for m in range(T):
        for n in range(T):
            want[m, n] = np.real(np.sum(qc[m] * np.conj(kc[n]) * np.exp(1j * (m - n) * th)))
    np.testing.assert_allclose(got, want, atol=1e-12)


def test_rejects_bad_arguments():
    x = np.zeros((8, 1, 8))
    with pytest.raises(ValueError):
        orc.rope3d(x, [(2, 2, 2)], [0, 8], (3, 3, 2))      # odd split
    with pytest.raises(ValueError):
        orc.rope3d(x, [(2, 2, 2)], [0, 8], (2, 2, 2))      # does not sum to head_dim
    with pytest.raises(ValueError):
        orc.rope3d(x, [(2, 2, 3)], [0, 8], (4, 2, 2))      # grid does not match length
