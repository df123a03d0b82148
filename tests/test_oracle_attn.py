"""Pins for the oracle's attention forward and backward (CPU only)."""
import math

import numpy as np
import pytest

from oracle import vfm_oracle as orc


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _inputs(cu, H, D, seed):
    n = cu[-1]
    return (_rand((n, H, D), seed), _rand((n, H, D), seed + 1), _rand((n, H, D), seed + 2),
            _rand((n, H, D), seed + 3))


# ---------------------------------------------------------------- closed forms
def test_single_token_segment_returns_v():
    cu = [0, 1, 2, 2, 3]                       # three 1-token segments and an empty one
    q, k, v, do = _inputs(cu, 2, 8, 0)
    scale = 0.37
    out, lse = orc.attn_fwd(q, k, v, cu, scale)
    np.testing.assert_array_equal(out, v)
    np.testing.assert_allclose(lse.T, scale * (q * k).sum(-1), rtol=1e-14)
    dq, dk, dv = orc.attn_bwd(q, k, v, do, cu, scale)
    np.testing.assert_array_equal(dv, do)
    np.testing.assert_allclose(dq, 0, atol=1e-14)      # dS = P (dP - Delta) = 0 up to rounding
    np.testing.assert_allclose(dk, 0, atol=1e-14)


def test_zero_queries_give_segment_mean():
    cu = [0, 5, 12]
    q, k, v, do = _inputs(cu, 2, 8, 10)
    q[:] = 0
    out, lse = orc.attn_fwd(q, k, v, cu, 0.5)
    dq, dk, dv = orc.attn_bwd(q, k, v, do, cu, 0.5)
    for a, b in ((0, 5), (5, 12)):
        np.testing.assert_allclose(out[a:b], np.broadcast_to(v[a:b].mean(0), out[a:b].shape), atol=1e-14)
        np.testing.assert_allclose(lse[:, a:b], math.log(b - a), atol=1e-14)
        np.testing.assert_allclose(dv[a:b], np.broadcast_to(do[a:b].sum(0) / (b - a), dv[a:b].shape), atol=1e-14)
    np.testing.assert_allclose(dk, 0, atol=1e-14)


def test_two_keys_is_logistic():
    # softmax over two keys is the logistic function of the score difference
    q, k, v, _ = _inputs([0, 2], 1, 4, 20)
    scale = 0.8
    out, lse = orc.attn_fwd(q, k, v, [0, 2], scale)
    for i in range(2):
        s0 = scale * float(q[i, 0] @ k[0, 0])
        s1 = scale * float(q[i, 0] @ k[1, 0])
        p0 = 1.0 / (1.0 + math.exp(s1 - s0))
        np.testing.assert_allclose(out[i, 0], p0 * v[0, 0] + (1 - p0) * v[1, 0], atol=1e-14)
        assert abs(lse[0, i] - math.log(math.exp(s0) + math.exp(s1))) < 1e-13


def test_rows_of_p_sum_to_one_and_v_shift():
    cu = [0, 7, 20]
    q, k, v, _ = _inputs(cu, 3, 8, 30)
    out1, _ = orc.attn_fwd(q, k, np.ones_like(v), cu, 0.4)
    np.testing.assert_allclose(out1, 1.0, atol=1e-14)
    out, _ = orc.attn_fwd(q, k, v, cu, 0.4)
    out_s, _ = orc.attn_fwd(q, k, v + 2.5, cu, 0.4)
    np.testing.assert_allclose(out_s, out + 2.5, atol=1e-13)


def test_lse_naive_and_stable():
    cu = [0, 6]
    q, k, v, _ = _inputs(cu, 1, 4, 40)
    _, lse = orc.attn_fwd(q, k, v, cu, 0.3)
    naive = np.log(np.exp(0.3 * q[:, 0] @ k[:, 0].T).sum(1))
    np.testing.assert_allclose(lse[0], naive, rtol=1e-13)
    out, lse = orc.attn_fwd(50 * q, 50 * k, v, cu, 0.3)      # scores in the thousands
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))


# ------------------------------------------------------------------ invariants
def test_packed_equals_each_clip_alone():
    lens = [5, 1, 9, 0, 4]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k, v, do = _inputs(cu, 2, 8, 50)
    out, lse = orc.attn_fwd(q, k, v, cu, 0.35)
    dq, dk, dv = orc.attn_bwd(q, k, v, do, cu, 0.35)
    for a, b in zip(cu[:-1], cu[1:]):
        if a == b:
            continue
        sl = slice(a, b)
        o1, l1 = orc.attn_fwd(q[sl], k[sl], v[sl], [0, b - a], 0.35)
        g1 = orc.attn_bwd(q[sl], k[sl], v[sl], do[sl], [0, b - a], 0.35)
        np.testing.assert_allclose(out[sl], o1, atol=1e-14)
        np.testing.assert_allclose(lse[:, sl], l1, atol=1e-14)
        for full, alone in zip((dq, dk, dv), g1):
            np.testing.assert_allclose(full[sl], alone, atol=1e-13)


def test_other_clips_do_not_leak():
    cu = [0, 6, 14]
    q, k, v, do = _inputs(cu, 2, 8, 60)
    out, _ = orc.attn_fwd(q, k, v, cu, 0.3)
    k2, v2 = k.copy(), v.copy()
    k2[6:] += 3.0
    v2[6:] -= 7.0
    out2, _ = orc.attn_fwd(q, k2, v2, cu, 0.3)
    np.testing.assert_array_equal(out2[:6], out[:6])
    assert not np.allclose(out2[6:], out[6:])


def test_key_shift_invariance_means_dk_sums_to_zero():
    cu = [0, 9, 15]
    q, k, v, do = _inputs(cu, 2, 8, 70)
    _, dk, _ = orc.attn_bwd(q, k, v, do, cu, 0.3)
    np.testing.assert_allclose(dk[0:9].sum(0), 0, atol=1e-13)
    np.testing.assert_allclose(dk[9:15].sum(0), 0, atol=1e-13)
    assert np.abs(dk).max() > 1e-3


def test_key_value_permutation():
    cu = [0, 11]
    q, k, v, do = _inputs(cu, 2, 8, 80)
    perm = np.random.default_rng(1).permutation(11)
    out, lse = orc.attn_fwd(q, k, v, cu, 0.3)
    dq, dk, dv = orc.attn_bwd(q, k, v, do, cu, 0.3)
    out_p, lse_p = orc.attn_fwd(q, k[perm], v[perm], cu, 0.3)
    dq_p, dk_p, dv_p = orc.attn_bwd(q, k[perm], v[perm], do, cu, 0.3)
    np.testing.assert_allclose(out_p, out, atol=1e-14)
    np.testing.assert_allclose(lse_p, lse, atol=1e-14)
    np.testing.assert_allclose(dq_p, dq, atol=1e-13)
    np.testing.assert_allclose(dk_p, dk[perm], atol=1e-13)
    np.testing.assert_allclose(dv_p, dv[perm], atol=1e-13)


# ------------------------------------------------------- independent opinions
def _brute_dense(q, k, v, cu, scale):
    """Dense total x total scores with an explicit block-diagonal mask, Python loops."""
    n, H, D = q.shape
    seg = [0] * n
    for s in range(len(cu) - 1):
        for t in range(cu[s], cu[s + 1]):
            seg[t] = s
    out = np.zeros((n, H, D))
    lse = np.zeros((H, n))
    for h in range(H):
        for i in range(n):
            scores = []
            for j in range(n):
                if seg[i] != seg[j]:
                    scores.append(-math.inf)
                else:
                    scores.append(scale * sum(q[i, h, d] * k[j, h, d] for d in range(D)))
            z = sum(math.exp(s) for s in scores)
            lse[h, i] = math.log(z)
            for j in range(n):
                p = math.exp(scores[j]) / z
                for d in range(D):
                    out[i, h, d] += p * v[j, h, d]
    return out, lse


def test_forward_against_dense_masked_brute_force():
    cu = [0, 3, 3, 8, 9]
    q, k, v, _ = _inputs(cu, 2, 4, 90)
    out, lse = orc.attn_fwd(q, k, v, cu, 0.6)
    bo, bl = _brute_dense(q, k, v, cu, 0.6)
    np.testing.assert_allclose(out, bo, atol=1e-13)
    np.testing.assert_allclose(lse, bl, atol=1e-13)


def test_gradients_against_central_differences():
    # the tiny configuration: 32 tokens, 2 heads, head_dim 64, scale 1/8
    from paper_2503_12964_amd import workloads as W
    wl = W.WORKLOADS["C1"]
    shape = (wl.total_tokens, wl.n_heads, wl.head_dim)
    q, k, v, do = (W.normal_f32(0, n, shape).astype(np.float64) for n in ("q", "k", "v", "dout"))
    cu, scale, eps = wl.cu_seqlens, 0.125, 1e-5
    grads = orc.attn_bwd(q, k, v, do, cu, scale)

    def loss(q_, k_, v_):
        return float((orc.attn_fwd(q_, k_, v_, cu, scale)[0] * do).sum())

    rng = np.random.default_rng(0)
    for which, g in enumerate(grads):
        idx = {tuple(rng.integers(0, s) for s in shape) for _ in range(40)}
        num = []
        for ix in idx:
            args = [q.copy(), k.copy(), v.copy()]
            args[which][ix] += eps
            up = loss(*args)
            args[which][ix] -= 2 * eps
            num.append((up - loss(*args)) / (2 * eps))
        ana = np.array([g[ix] for ix in idx])
        num = np.array(num)
        assert np.linalg.norm(num - ana) <= 1e-7 * np.linalg.norm(ana)


def test_gradients_full_jacobian_tiny():
    # every element, two segments, so a wrong index anywhere shows
    cu = [0, 3, 7]
    q, k, v, do = _inputs(cu, 2, 4, 100)
    scale, eps = 0.7, 1e-6
    grads = orc.attn_bwd(q, k, v, do, cu, scale)
    base = [q, k, v]
    for which in range(3):
        num = np.zeros_like(q)
        for ix in np.ndindex(*q.shape):
            args = [a.copy() for a in base]
            args[which][ix] += eps
            up = (orc.attn_fwd(*args, cu, scale)[0] * do).sum()
            args[which][ix] -= 2 * eps
            num[ix] = (up - (orc.attn_fwd(*args, cu, scale)[0] * do).sum()) / (2 * eps)
        np.testing.assert_allclose(grads[which], num, atol=2e-8)


def test_against_torch_autograd_fp64():
    torch = pytest.importorskip("torch")
    lens = [40, 1, 25]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k, v, do = _inputs(cu, 3, 16, 110)
    scale = 0.25
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    seg = torch.tensor(np.repeat(np.arange(len(lens)), lens))
    mask = seg[:, None] == seg[None, :]
    s = torch.einsum("ihd,jhd->hij", tq, tk) * scale
    s = s.masked_fill(~mask[None], float("-inf"))
    o = torch.einsum("hij,jhd->ihd", torch.softmax(s, dim=-1), tv)
    (o * torch.tensor(do)).sum().backward()
    out, lse = orc.attn_fwd(q, k, v, cu, scale)
    dq, dk, dv = orc.attn_bwd(q, k, v, do, cu, scale)
    np.testing.assert_allclose(out, o.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-13)


# ---------------------------------------------------------- Delta from a handed-over out
def test_backward_with_the_forwards_own_out_is_the_exact_gradient():
    lens = [9, 0, 5, 1]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k, v, do = _inputs(cu, 3, 8, 130)
    out, _ = orc.attn_fwd(q, k, v, cu, 0.4)
    for a, b in zip(orc.attn_bwd(q, k, v, do, cu, 0.4), orc.attn_bwd(q, k, v, do, cu, 0.4, out=out)):
        np.testing.assert_allclose(a, b, atol=1e-15)
    with pytest.raises(ValueError):
        orc.attn_bwd(q, k, v, do, cu, 0.4, out=out[:, :2])


def test_a_perturbed_out_moves_the_gradients_through_delta_alone():
    # Closed form, written with plain loops: with out + E handed over, Delta_i grows by
    # e_i = sum_d dO_id E_id, hence dS_ij falls by P_ij e_i:
    #   dQ_i falls by scale * e_i * sum_j P_ij K_j,  dK_j by scale * sum_i P_ij e_i Q_i,  dV is unchanged.
    lens = [6, 4]
    cu = np.concatenate([[0], np.cumsum(lens)])
    H, D, scale = 2, 4, 0.7
    q, k, v, do = _inputs(cu, H, D, 131)
    out, _ = orc.attn_fwd(q, k, v, cu, scale)
    E = 0.05 * np.random.default_rng(132).standard_normal(out.shape)
    base = orc.attn_bwd(q, k, v, do, cu, scale)
    moved = orc.attn_bwd(q, k, v, do, cu, scale, out=out + E)
    want_dq, want_dk = np.zeros_like(q), np.zeros_like(k)
    for s in range(len(lens)):
        a, b = int(cu[s]), int(cu[s + 1])
        for h in range(H):
            for i in range(a, b):
                w = np.array([np.exp(scale * float(q[i, h] @ k[j, h])) for j in range(a, b)])
                p = w / w.sum()
                e = float(do[i, h] @ E[i, h])
                for jj, j in enumerate(range(a, b)):
                    want_dq[i, h] -= scale * e * p[jj] * k[j, h]
                    want_dk[j, h] -= scale * e * p[jj] * q[i, h]
    np.testing.assert_allclose(moved[0] - base[0], want_dq, atol=1e-13)
    np.testing.assert_allclose(moved[1] - base[1], want_dk, atol=1e-13)
    np.testing.assert_allclose(moved[2], base[2], atol=1e-15)


# ---------------------------------------------------------- row-subset helpers
def test_row_helpers_match_full_functions():
    lens = [13, 0, 6, 21]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k, v, do = _inputs(cu, 2, 8, 120)
    out, lse = orc.attn_fwd(q, k, v, cu, 0.3)
    dq, dk, dv = orc.attn_bwd(q, k, v, do, cu, 0.3)
    rows = np.array([0, 12, 13, 18, 19, 39, 5])
    o_r, l_r = orc.attn_fwd_rows(q, k, v, cu, 0.3, 1, rows)
    np.testing.assert_allclose(o_r, out[rows, 1], atol=1e-14)
    np.testing.assert_allclose(l_r, lse[1, rows], atol=1e-14)
    dq_r, _, _ = orc.attn_bwd_rows(q, k, v, do, cu, 0.3, 1, rows)
    np.testing.assert_allclose(dq_r, dq[rows, 1], atol=1e-14)
    # a partition of all rows rebuilds dK and dV
    dk_sum = np.zeros((cu[-1], 8))
    dv_sum = np.zeros((cu[-1], 8))
    for part in np.array_split(np.random.default_rng(3).permutation(cu[-1]), 4):
        _, dkp, dvp = orc.attn_bwd_rows(q, k, v, do, cu, 0.3, 1, part)
        dk_sum += dkp
        dv_sum += dvp
    np.testing.assert_allclose(dk_sum, dk[:, 1], atol=1e-13)
    np.testing.assert_allclose(dv_sum, dv[:, 1], atol=1e-13)


def test_column_helper_matches_full_function():
    lens = [9, 30, 4]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k, v, do = _inputs(cu, 2, 8, 130)
    _, dk, dv = orc.attn_bwd(q, k, v, do, cu, 0.3)
    cols = np.array([9, 17, 38, 22])
    dk_c, dv_c = orc.attn_bwd_cols(q, k, v, do, cu, 0.3, 1, cols, row_chunk=7)
    np.testing.assert_allclose(dk_c, dk[cols, 1], atol=1e-13)
    np.testing.assert_allclose(dv_c, dv[cols, 1], atol=1e-13)
    with pytest.raises(ValueError):
        orc.attn_bwd_cols(q, k, v, do, cu, 0.3, 1, [3, 20])


def test_bad_cu_seqlens_rejected():
    q = np.zeros((4, 1, 2))
    for cu in ([1, 4], [0, 3], [0, 3, 2, 4]):
        with pytest.raises(ValueError):
            orc.attn_fwd(q, q, q, cu, 1.0)
