"""Pins for the oracle's temporal attention (one sequence per pixel across frames, Section 4.6)
and its gradients (CPU only)."""
import numpy as np

from oracle import vfm_oracle as orc

GRIDS = [(3, 2, 2), (1, 1, 3), (0, 1, 1), (5, 1, 2)]
CU = np.concatenate([[0], np.cumsum([t * h * w for t, h, w in GRIDS])])
TOTAL = int(CU[-1])
H, D = 2, 8
SCALE = 0.4


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _pixel_major():
    """Permutation that makes every temporal sequence contiguous, and its boundaries."""
    perm, lens = [], []
    for s, (T, Hh, W) in enumerate(GRIDS):
        for p in range(Hh * W):
            perm += [int(CU[s]) + t * Hh * W + p for t in range(T)]
            if T:
                lens.append(T)
    return np.array(perm), np.concatenate([[0], np.cumsum(lens)])


def test_equals_packed_attention_on_the_gathered_layout():
    q, k, v, do = (_rand((TOTAL, H, D), s) for s in range(4))
    perm, cu_t = _pixel_major()
    out = orc.temporal_attn_fwd(q, k, v, GRIDS, CU, SCALE)
    want, _ = orc.attn_fwd(q[perm], k[perm], v[perm], cu_t, SCALE)
    np.testing.assert_allclose(out[perm], want, rtol=0, atol=1e-14)
    got = orc.temporal_attn_bwd(q, k, v, do, GRIDS, CU, SCALE)
    ref = orc.attn_bwd(q[perm], k[perm], v[perm], do[perm], cu_t, SCALE)
    for a, b in zip(got, ref):
        np.testing.assert_allclose(a[perm], b, rtol=0, atol=1e-13)


def test_single_frame_clip_returns_values():
    q, k, v = (_rand((TOTAL, H, D), s) for s in range(3))
    out = orc.temporal_attn_fwd(q, k, v, GRIDS, CU, SCALE)
    a, b = int(CU[1]), int(CU[2])           # the (1,1,3) clip: three sequences of one token
    np.testing.assert_allclose(out[a:b], v[a:b], rtol=0, atol=1e-15)


def test_zero_queries_average_the_pixel_over_frames():
    k, v = _rand((TOTAL, H, D), 5), _rand((TOTAL, H, D), 6)
    out = orc.temporal_attn_fwd(np.zeros((TOTAL, H, D)), k, v, GRIDS, CU, SCALE)
    a = int(CU[3])                           # the (5,1,2) clip: pixel p has rows a + 2t + p
    for p in range(2):
        rows = a + 2 * np.arange(5) + p
        np.testing.assert_allclose(out[rows], np.broadcast_to(v[rows].mean(axis=0), (5, H, D)), rtol=0, atol=1e-14)


def test_pixels_do_not_mix():
    q, k, v = (_rand((TOTAL, H, D), s) for s in range(7, 10))
    out = orc.temporal_attn_fwd(q, k, v, GRIDS, CU, SCALE)
    k2, v2 = k.copy(), v.copy()
    rows_other = np.arange(3) * 4 + 1        # pixel 1 of the (3,2,2) clip
    k2[rows_other] += 3.0
    v2[rows_other] -= 2.0
    out2 = orc.temporal_attn_fwd(q, k2, v2, GRIDS, CU, SCALE)
    rows_p0 = np.arange(3) * 4               # pixel 0 is unaffected
    np.testing.assert_array_equal(out[rows_p0], out2[rows_p0])
    assert np.max(np.abs(out[rows_other] - out2[rows_other])) > 0.1


def test_gradients_match_central_differences():
    grids, cu = [(3, 1, 2)], np.array([0, 6])
    q, k, v, do = (_rand((6, 1, 4), s) for s in range(10, 14))
    grads = orc.temporal_attn_bwd(q, k, v, do, grids, cu, SCALE)

    def loss(qq, kk, vv):
        return float(np.sum(orc.temporal_attn_fwd(qq, kk, vv, grids, cu, SCALE) * do))

    h = 1e-6
    for which, (x, g) in enumerate(zip((q, k, v), grads)):
        num = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            args_p, args_m = [q, k, v], [q, k, v]
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            args_p[which], args_m[which] = xp, xm
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * h)
        np.testing.assert_allclose(g, num, rtol=1e-6, atol=1e-8)
