"""Pins for the oracle's packed cross-attention (video queries x text keys/values) and its
gradients (CPU only): reduction to self-attention, closed forms, independence of packed
sequences, key permutation, brute-force loops, finite differences, torch fp64 autograd."""
import numpy as np
import pytest

from oracle import vfm_oracle as orc

CU_Q = np.array([0, 7, 7, 19, 24])      # sequence 1 has no queries
CU_KV = np.array([0, 3, 5, 6, 15])      # ... but two keys; sequence 2 has a single key
H, D = 2, 8
SCALE = 0.3


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _inputs(seed=0):
    return (_rand((24, H, D), seed), _rand((15, H, D), seed + 1), _rand((15, H, D), seed + 2),
            _rand((24, H, D), seed + 3))


def test_equal_ranges_reduce_to_self_attention():
    cu = np.array([0, 5, 5, 11, 16])
    q, k, v, do = (_rand((16, H, D), s) for s in range(4))
    o1, l1 = orc.xattn_fwd(q, k, v, cu, cu, SCALE)
    o2, l2 = orc.attn_fwd(q, k, v, cu, SCALE)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(l1, l2, rtol=0, atol=1e-14)
    for a, b in zip(orc.xattn_bwd(q, k, v, do, cu, cu, SCALE), orc.attn_bwd(q, k, v, do, cu, SCALE)):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_single_key_returns_its_value_for_every_query():
    q, k, v, do = _inputs()
    out, lse = orc.xattn_fwd(q, k, v, CU_Q, CU_KV, SCALE)
    for h in range(H):
        np.testing.assert_allclose(out[7:19, h], np.broadcast_to(v[5, h], (12, D)), rtol=0, atol=1e-15)
        np.testing.assert_allclose(lse[h, 7:19], SCALE * q[7:19, h] @ k[5, h], rtol=0, atol=1e-14)
    dq, dk, dv = orc.xattn_bwd(q, k, v, do, CU_Q, CU_KV, SCALE)
    # softmax over one key is constant: no gradient reaches q or that key; dV collects all dO
    # (dS = P (dP - Delta) with P = 1 and Delta = dP up to rounding)
    assert np.max(np.abs(dq[7:19])) < 1e-14 and np.max(np.abs(dk[5])) < 1e-13
    np.testing.assert_allclose(dv[5], do[7:19].sum(axis=0), rtol=0, atol=1e-13)


def test_zero_queries_give_mean_value_and_log_count():
    q, k, v, do = _inputs(4)
    out, lse = orc.xattn_fwd(np.zeros_like(q), k, v, CU_Q, CU_KV, SCALE)
    np.testing.assert_allclose(out[19:24], np.broadcast_to(v[6:15].mean(axis=0), (5, H, D)), rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse[:, 19:24], np.log(9.0), rtol=0, atol=1e-14)


def test_keys_without_queries_get_zero_gradients():
    q, k, v, do = _inputs(5)
    _, dk, dv = orc.xattn_bwd(q, k, v, do, CU_Q, CU_KV, SCALE)
    assert np.all(dk[3:5] == 0) and np.all(dv[3:5] == 0)


def test_packed_equals_each_sequence_alone():
    q, k, v, do = _inputs(6)
    out, lse = orc.xattn_fwd(q, k, v, CU_Q, CU_KV, SCALE)
    dq, dk, dv = orc.xattn_bwd(q, k, v, do, CU_Q, CU_KV, SCALE)
    for s in (0, 2, 3):
        a, b, c, d = CU_Q[s], CU_Q[s + 1], CU_KV[s], CU_KV[s + 1]
        o1, l1 = orc.xattn_fwd(q[a:b], k[c:d], v[c:d], [0, b - a], [0, d - c], SCALE)
        g1 = orc.xattn_bwd(q[a:b], k[c:d], v[c:d], do[a:b], [0, b - a], [0, d - c], SCALE)
        np.testing.assert_allclose(out[a:b], o1, rtol=0, atol=1e-14)
        np.testing.assert_allclose(lse[:, a:b], l1, rtol=0, atol=1e-14)
        np.testing.assert_allclose(dq[a:b], g1[0], rtol=0, atol=1e-13)
        np.testing.assert_allclose(dk[c:d], g1[1], rtol=0, atol=1e-13)
        np.testing.assert_allclose(dv[c:d], g1[2], rtol=0, atol=1e-13)


def test_key_permutation_invariance():
    q, k, v, do = _inputs(7)
    perm = np.arange(15)
    perm[6:15] = 6 + np.random.default_rng(1).permutation(9)
    o1, l1 = orc.xattn_fwd(q, k, v, CU_Q, CU_KV, SCALE)
    o2, l2 = orc.xattn_fwd(q, k[perm], v[perm], CU_Q, CU_KV, SCALE)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(l1, l2, rtol=0, atol=1e-14)
    g1 = orc.xattn_bwd(q, k, v, do, CU_Q, CU_KV, SCALE)
    g2 = orc.xattn_bwd(q, k[perm], v[perm], do, CU_Q, CU_KV, SCALE)
    np.testing.assert_allclose(g1[0], g2[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(g1[1][perm], g2[1], rtol=0, atol=1e-13)
    np.testing.assert_allclose(g1[2][perm], g2[2], rtol=0, atol=1e-13)


def test_forward_against_plain_loops():
    q, k, v, _ = _inputs(8)
    out, lse = orc.xattn_fwd(q, k, v, CU_Q, CU_KV, SCALE)
    for s in range(4):
        for i in range(CU_Q[s], CU_Q[s + 1]):
            for h in range(H):
                w = [np.exp(SCALE * sum(q[i, h, d] * k[j, h, d] for d in range(D)))
                     for j in range(CU_KV[s], CU_KV[s + 1])]
                z = sum(w)
                want = sum(wj / z * v[j, h] for wj, j in zip(w, range(CU_KV[s], CU_KV[s + 1])))
                np.testing.assert_allclose(out[i, h], want, rtol=0, atol=1e-13)
                assert abs(lse[h, i] - np.log(z)) < 1e-13


def test_gradients_match_central_differences():
    cq, ck = np.array([0, 3, 5]), np.array([0, 4, 6])
    q, k, v, do = _rand((5, 1, 4), 0), _rand((6, 1, 4), 1), _rand((6, 1, 4), 2), _rand((5, 1, 4), 3)
    grads = orc.xattn_bwd(q, k, v, do, cq, ck, SCALE)

    def loss(qq, kk, vv):
        return float(np.sum(orc.xattn_fwd(qq, kk, vv, cq, ck, SCALE)[0] * do))

    h = 1e-6
    for which, (x, g) in enumerate(zip((q, k, v), grads)):
        num = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            args_p = [q, k, v]
            args_m = [q, k, v]
            args_p[which], args_m[which] = xp, xm
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * h)
        np.testing.assert_allclose(g, num, rtol=1e-6, atol=1e-8)


def test_against_torch_autograd():
    torch = pytest.importorskip("torch")
    q, k, v, do = _inputs(9)
    qt, kt, vt = (torch.tensor(x, requires_grad=True) for x in (q, k, v))
    outs = []
    for s in range(4):
        a, b, c, d = int(CU_Q[s]), int(CU_Q[s + 1]), int(CU_KV[s]), int(CU_KV[s + 1])
        if b == a:
            continue
        att = torch.softmax(SCALE * torch.einsum("ihd,jhd->hij", qt[a:b], kt[c:d]), dim=-1)
        outs.append(torch.einsum("hij,jhd->ihd", att, vt[c:d]))
    ot = torch.cat(outs, dim=0)
    (ot * torch.tensor(do)).sum().backward()
    out, _ = orc.xattn_fwd(q, k, v, CU_Q, CU_KV, SCALE)
    dq, dk, dv = orc.xattn_bwd(q, k, v, do, CU_Q, CU_KV, SCALE)
    np.testing.assert_allclose(out, ot.detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dq, qt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, kt.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, vt.grad.numpy(), rtol=0, atol=1e-12)


def test_queries_without_keys_are_rejected():
    q, k, v, _ = _inputs(10)
    with pytest.raises(ValueError):
        orc.xattn_fwd(q, k, v, [0, 7, 24], [0, 15, 15], SCALE)
