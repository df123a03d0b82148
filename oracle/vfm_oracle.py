"""fp64 CPU oracle for packed 3D-RoPE self-attention (forward and backward).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference the GPU
library is judged against.  Only the tests, the smoke check and the
cpu_baseline leg of the benchmark may import it; the product path never does.
It shares no code with the HIP kernels and imports nothing from the package.

Everything is numpy float64.  Inputs are widened exactly (a bf16 or fp32 bit
pattern is representable in fp64), so input quantisation is never charged as
error.  Each function writes the plain definition out; there is no tiling,
no online softmax, no fusion.  A matmul (numpy `@`) is used as a library step.

What the paper fixes, and where:
  * Section 3.1 (dataset preparation and blending): clips of different
    shapes are concatenated along the sequence dimension with micro-batch 1
    ("sequence packing"), so the packed layout is [total_tokens, heads,
    head_dim] with segment boundaries cu_seqlens, and attention never crosses
    a boundary.
  * Section 4.2 (training pipeline): the 3D latent tokens of a clip are
    flattened into one sequence of spacetime patches.  Section 4.6 gives the
    flattened shape [b, h*w*t, d] and notes that spatial attention views the
    same buffer as [(b*t), h*w, d]; that view is free only when t is the
    slowest-varying index, hence r = (t*H + h)*W + w here.
  * Section 4.4 (context parallel paragraph) and Section 4.6: every query
    token is computed against the keys and values of all tokens of its own
    sequence -- full, bidirectional attention, no causal mask.
  * Section 5.2 and Table 1: multi-head attention, one K/V head per Q head,
    head_dim = hidden / heads = 128.

  * Section 4.5.1 (paragraph on QK normalisation): Q and K are normalised
    per attention head (not over the whole hidden dimension) right before
    the dot-product attention.

What the paper does not fix (readings taken; all are restated in the design
notes of the repository): the rotary embedding itself (theta, per-axis
split, adjacent-pair convention, per-axis frequency exponent, integer grid
positions starting at 0), the softmax scale (an argument), natural-log
units for the log-sum-exp, and the kind of per-head normalisation (taken as
root-mean-square normalisation with a learned gain of head_dim entries shared
by all heads, and an epsilon inside the square root).

Pins (tests/test_oracle_*.py): single-token segment returns V; Q = 0 returns
the segment mean of V and lse = ln N; packed equals per-clip; RoPE keeps
norms, is the identity at the origin, inverts exactly, is shift-invariant in
the scores, and reduces to textbook complex-number 1-D RoPE; softmax row
sums; sum of dK over a segment is zero; key/value permutation invariance;
central finite differences; a dense masked brute force written with Python
loops; PyTorch fp64 autograd as a third opinion.  tests/oracle_mutants.py
plants some fifty single mistakes in a copy of this file (dropped terms and
factors, wrong signs, indices and axes, transposed operands) and
tests/test_oracle_mutations.py checks that the pins reject each of them.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "token_coords",
    "rope3d",
    "qknorm_rope3d",
    "qknorm_rope3d_bwd",
    "attn_fwd",
    "attn_bwd",
    "xattn_fwd",
    "xattn_bwd",
    "temporal_attn_fwd",
    "temporal_attn_bwd",
    "fp8_e4m3_decode",
    "fp8_e4m3_encode",
    "fp8_tile_exponent",
    "attn_fwd_rows",
    "attn_bwd_rows",
    "attn_bwd_cols",
]


def _as_f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def _check_cu(cu_seqlens, total_tokens: int) -> np.ndarray:
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    if cu.ndim != 1 or cu.size < 1 or cu[0] != 0 or cu[-1] != total_tokens:
        raise ValueError("cu_seqlens must start at 0 and end at total_tokens")
    if np.any(np.diff(cu) < 0):
        raise ValueError("cu_seqlens must be non-decreasing")
    return cu


def token_coords(thw, cu_seqlens) -> np.ndarray:
    """(t, h, w) grid position of every packed token.

    Section 4.2 / 4.6: a clip with latent grid (T, H, W) is flattened with t
    slowest and w fastest.  Packed token n of segment s has local index
    r = n - cu[s] and position t = r // (H*W), h = (r // W) % H, w = r % W.
    Returns int64 [total_tokens, 3].
    """
    thw = np.asarray(thw, dtype=np.int64).reshape(-1, 3)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    if thw.shape[0] != cu.size - 1:
        raise ValueError("one (T,H,W) triple per segment")
    total = int(cu[-1])
    pos = np.zeros((total, 3), dtype=np.int64)
    for s in range(thw.shape[0]):
        T, H, W = (int(v) for v in thw[s])
        a, b = int(cu[s]), int(cu[s + 1])
        if T * H * W != b - a:
            raise ValueError(f"segment {s}: T*H*W != segment length")
        r = np.arange(b - a, dtype=np.int64)
        pos[a:b, 0] = r // (H * W)
        pos[a:b, 1] = (r // W) % H
        pos[a:b, 2] = r % W
    return pos


def rope3d(x, thw, cu_seqlens, dims, theta: float = 10000.0,
           inverse: bool = False, pos_offset=(0, 0, 0)) -> np.ndarray:
    """3D rotary position embedding of x[total, heads, head_dim] (fp64 copy).

    The head vector is cut into three contiguous slices of widths
    dims = (d_t, d_h, d_w), d_t + d_h + d_w = head_dim, all even.  Slice A is
    an ordinary 1-D rotary embedding driven by the token's position along
    axis A: for i in [0, d_A/2) the adjacent pair (x[o_A+2i], x[o_A+2i+1]) is
    rotated by the angle  phi = pos_A * theta**(-2i/d_A):
        x0' = x0 cos(phi) - x1 sin(phi),   x1' = x0 sin(phi) + x1 cos(phi).
    inverse=True rotates by -phi (the transpose, used for gradients).
    pos_offset shifts every position by a constant (only tests use it, to
    check that scores depend on position differences alone).
    """
    x = _as_f64(x)
    total, _, D = x.shape
    d_t, d_h, d_w = (int(d) for d in dims)
    if d_t + d_h + d_w != D or any(d % 2 for d in (d_t, d_h, d_w)):
        raise ValueError("dims must be even and sum to head_dim")
    _check_cu(cu_seqlens, total)
    pos = token_coords(thw, cu_seqlens) + np.asarray(pos_offset, dtype=np.int64)
    y = x.copy()
    start = 0
    for axis, d_a in enumerate((d_t, d_h, d_w)):
        if d_a == 0:
            continue
        i = np.arange(d_a // 2, dtype=np.float64)
        freq = float(theta) ** (-2.0 * i / d_a)                    # [d_a/2]
        phi = pos[:, axis].astype(np.float64)[:, None] * freq[None, :]
        if inverse:
            phi = -phi
        c = np.cos(phi)[:, None, :]                                # [total,1,d_a/2]
        s = np.sin(phi)[:, None, :]
        x0 = x[:, :, start:start + d_a:2]
        x1 = x[:, :, start + 1:start + d_a:2]
        y[:, :, start:start + d_a:2] = x0 * c - x1 * s
        y[:, :, start + 1:start + d_a:2] = x0 * s + x1 * c
        start += d_a
    return y


def _rstd(x: np.ndarray, eps: float) -> np.ndarray:
    """1 / sqrt(mean_d x_d^2 + eps) per (token, head), shape [total, heads, 1]."""
    return 1.0 / np.sqrt(np.mean(x * x, axis=2, keepdims=True) + float(eps))


def qknorm_rope3d(x, gain, eps: float, thw, cu_seqlens, dims, theta: float = 10000.0) -> np.ndarray:
    """Per-head normalisation of x[total, heads, head_dim] followed by 3D RoPE.

    Section 4.5.1 normalises Q and K per head before attention; the reading
    taken is RMS normalisation with a learned gain g[head_dim]:
        r   = 1 / sqrt(mean_d x_d^2 + eps)          per (token, head)
        z_d = x_d * r * g_d
        y   = rope3d(z)
    Returns y (fp64).
    """
    x = _as_f64(x)
    g = np.asarray(gain, dtype=np.float64)
    if g.shape != (x.shape[2],):
        raise ValueError("gain must have head_dim entries")
    z = x * _rstd(x, eps) * g[None, None, :]
    return rope3d(z, thw, cu_seqlens, dims, theta)


def qknorm_rope3d_bwd(x, gain, eps: float, dy, thw, cu_seqlens, dims, theta: float = 10000.0):
    """Gradients of qknorm_rope3d with respect to x and the gain, given dy.

    With n = x r (the normalised vector), z = n g and y = R z (R the rotation,
    orthogonal):
        dz     = R^T dy                               (rotation by the negated angle)
        dgain  = sum over (token, head) of dz * n
        dn     = dz * g
        dx     = r * (dn - n * mean_d(dn_d n_d))      (Jacobian of x -> x r)
    Returns dx [total, heads, head_dim] and dgain [head_dim], both fp64.
    """
    x, dy = _as_f64(x), _as_f64(dy)
    g = np.asarray(gain, dtype=np.float64)
    r = _rstd(x, eps)
    n = x * r
    dz = rope3d(dy, thw, cu_seqlens, dims, theta, inverse=True)
    dgain = np.sum(dz * n, axis=(0, 1))
    dn = dz * g[None, None, :]
    dx = r * (dn - n * np.mean(dn * n, axis=2, keepdims=True))
    return dx, dgain


def _softmax_rows(S: np.ndarray):
    """Row softmax of a score matrix and its natural-log normaliser."""
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(axis=1, keepdims=True)
    return E / l, (m + np.log(l))[:, 0]


def attn_fwd(q, k, v, cu_seqlens, scale: float):
    """Packed multi-head self-attention forward.

    For each segment [a, b) and head h (Sections 3.1, 4.4, 4.6):
        S_ij = scale * sum_d Q_id K_jd           i, j in [a, b)
        P_ij = exp(S_ij) / sum_j' exp(S_ij')
        O_i  = sum_j P_ij V_j
        LSE_i = ln sum_j exp(S_ij)               (natural log)
    Returns out [total, heads, head_dim] and lse [heads, total], both fp64.
    Empty segments contribute nothing.
    """
    q, k, v = _as_f64(q), _as_f64(k), _as_f64(v)
    total, H, D = q.shape
    cu = _check_cu(cu_seqlens, total)
    out = np.zeros((total, H, D))
    lse = np.zeros((H, total))
    for s in range(cu.size - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        for h in range(H):
            S = scale * (q[a:b, h, :] @ k[a:b, h, :].T)
            P, L = _softmax_rows(S)
            out[a:b, h, :] = P @ v[a:b, h, :]
            lse[h, a:b] = L
    return out, lse


def attn_bwd(q, k, v, dout, cu_seqlens, scale: float, out=None):
    """Gradients of  sum(out * dout)  with respect to q, k, v.

    The softmax-attention gradient written out (no gradient flows into lse):
        Delta_i = sum_d dO_id O_id
        dV_j    = sum_i P_ij dO_i
        dP_ij   = sum_d dO_id V_jd
        dS_ij   = P_ij (dP_ij - Delta_i)
        dQ_i    = scale * sum_j dS_ij K_j
        dK_j    = scale * sum_i dS_ij Q_i
    P is recomputed from this module's own forward, and so is O: the result is
    the exact gradient.  The backward call of the method is handed the
    forward's output as an argument and forms Delta = rowsum(dO o O) from it;
    `out` (same shape as q), when given, takes that place in Delta and nowhere
    else, so that tests can tell the rounding of a handed-over bf16 `out`
    (which shows where dS cancels: peaky softmax, clips of a few tokens) from
    damage.  Returns dq, dk, dv with the shape of q, fp64.
    """
    q, k, v, dout = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(dout)
    total, H, D = q.shape
    cu = _check_cu(cu_seqlens, total)
    given = None if out is None else _as_f64(out)
    if given is not None and given.shape != q.shape:
        raise ValueError("out must have the shape of q")
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for s in range(cu.size - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        for h in range(H):
            Q, K, V, dO = q[a:b, h, :], k[a:b, h, :], v[a:b, h, :], dout[a:b, h, :]
            P, _ = _softmax_rows(scale * (Q @ K.T))
            O = P @ V if given is None else given[a:b, h, :]
            delta = (dO * O).sum(axis=1, keepdims=True)
            dv[a:b, h, :] = P.T @ dO
            dP = dO @ V.T
            dS = P * (dP - delta)
            dq[a:b, h, :] = scale * (dS @ K)
            dk[a:b, h, :] = scale * (dS.T @ Q)
    return dq, dk, dv


def xattn_fwd(q, k, v, cu_seqlens_q, cu_seqlens_kv, scale: float):
    """Packed multi-head cross-attention forward (Section 4.2: every transformer block
    attends from the video query tensor to the text embedding's keys and values).

    Sequence s owns queries [cu_q[s], cu_q[s+1]) of q[total_q, heads, head_dim] and keys /
    values [cu_kv[s], cu_kv[s+1]) of k, v[total_kv, heads, head_dim]:
        S_ij = scale * sum_d Q_id K_jd      i in the query range, j in the key range
        O_i  = sum_j softmax_j(S_ij) V_j,   LSE_i = ln sum_j exp(S_ij)
    A sequence with queries needs at least one key.  Returns out [total_q, heads, head_dim]
    and lse [heads, total_q], fp64.
    """
    q, k, v = _as_f64(q), _as_f64(k), _as_f64(v)
    total_q, H, D = q.shape
    cq = _check_cu(cu_seqlens_q, total_q)
    ck = _check_cu(cu_seqlens_kv, k.shape[0])
    if cq.size != ck.size:
        raise ValueError("cu_seqlens_q and cu_seqlens_kv must name the same number of sequences")
    out = np.zeros((total_q, H, D))
    lse = np.zeros((H, total_q))
    for s in range(cq.size - 1):
        a, b, c, d = int(cq[s]), int(cq[s + 1]), int(ck[s]), int(ck[s + 1])
        if b == a:
            continue
        if d == c:
            raise ValueError("a sequence with queries has no keys")
        for h in range(H):
            P, L = _softmax_rows(scale * (q[a:b, h, :] @ k[c:d, h, :].T))
            out[a:b, h, :] = P @ v[c:d, h, :]
            lse[h, a:b] = L
    return out, lse


def xattn_bwd(q, k, v, dout, cu_seqlens_q, cu_seqlens_kv, scale: float):
    """Gradients of  sum(out * dout)  of xattn_fwd with respect to q, k, v: the formulas of
    attn_bwd with i over the sequence's queries and j over its keys.  Keys of a sequence
    without queries get zero gradients.  Returns dq (shape of q), dk, dv (shape of k), fp64.
    """
    q, k, v, dout = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(dout)
    cq = _check_cu(cu_seqlens_q, q.shape[0])
    ck = _check_cu(cu_seqlens_kv, k.shape[0])
    if cq.size != ck.size:
        raise ValueError("cu_seqlens_q and cu_seqlens_kv must name the same number of sequences")
    H = q.shape[1]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for s in range(cq.size - 1):
        a, b, c, d = int(cq[s]), int(cq[s + 1]), int(ck[s]), int(ck[s + 1])
        if b == a:
            continue
        if d == c:
            raise ValueError("a sequence with queries has no keys")
        for h in range(H):
            Q, K, V, dO = q[a:b, h, :], k[c:d, h, :], v[c:d, h, :], dout[a:b, h, :]
            P, _ = _softmax_rows(scale * (Q @ K.T))
            delta = (dO * (P @ V)).sum(axis=1, keepdims=True)
            dS = P * (dO @ V.T - delta)
            dv[c:d, h, :] = P.T @ dO
            dq[a:b, h, :] = scale * (dS @ K)
            dk[c:d, h, :] = scale * (dS.T @ Q)
    return dq, dk, dv


def _temporal_rows(thw, cu_seqlens):
    """For every clip, the packed token rows of each temporal sequence: an int array
    [H*W, T] whose entry (p, t) is the row of pixel p in frame t (t is the slowest index of
    the flatten order)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    grids = np.asarray(thw, dtype=np.int64).reshape(-1, 3)
    for s, (T, H, W) in enumerate(grids):
        n = int(cu[s + 1] - cu[s])
        if n == 0:
            continue
        if T * H * W != n:
            raise ValueError("T*H*W must equal the clip length")
        yield int(cu[s]) + np.arange(T)[None, :] * (H * W) + np.arange(H * W)[:, None]


def temporal_attn_fwd(q, k, v, thw, cu_seqlens, scale: float):
    """Temporal attention of the spatial-temporal transformer (Section 4.6): attention among
    the inter-frame tokens of one pixel, i.e. the buffer [b, h*w*t, d] read as
    [(b*h*w), t, d].  For clip s with grid (T, H, W) and pixel p the sequence is the T rows
    cu[s] + t*H*W + p; within it, per head, out = softmax(scale Q K^T) V.
    Returns out [total, heads, head_dim], fp64.
    """
    q, k, v = _as_f64(q), _as_f64(k), _as_f64(v)
    _check_cu(cu_seqlens, q.shape[0])
    out = np.zeros_like(q)
    for rows in _temporal_rows(thw, cu_seqlens):
        Q, K, V = q[rows], k[rows], v[rows]                     # [pixels, T, heads, D]
        S = scale * np.einsum("pihd,pjhd->phij", Q, K)
        S -= S.max(axis=3, keepdims=True)
        P = np.exp(S)
        P /= P.sum(axis=3, keepdims=True)
        out[rows] = np.einsum("phij,pjhd->pihd", P, V)
    return out


def temporal_attn_bwd(q, k, v, dout, thw, cu_seqlens, scale: float):
    """Gradients of  sum(out * dout)  of temporal_attn_fwd with respect to q, k, v (the
    formulas of attn_bwd inside every temporal sequence)."""
    q, k, v, dout = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(dout)
    _check_cu(cu_seqlens, q.shape[0])
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for rows in _temporal_rows(thw, cu_seqlens):
        Q, K, V, dO = q[rows], k[rows], v[rows], dout[rows]
        S = scale * np.einsum("pihd,pjhd->phij", Q, K)
        S -= S.max(axis=3, keepdims=True)
        P = np.exp(S)
        P /= P.sum(axis=3, keepdims=True)
        O = np.einsum("phij,pjhd->pihd", P, V)
        delta = np.einsum("pihd,pihd->phi", dO, O)[..., None]
        dP = np.einsum("pihd,pjhd->phij", dO, V)
        dS = P * (dP - delta)
        dv[rows] = np.einsum("phij,pihd->pjhd", P, dO)
        dq[rows] = scale * np.einsum("phij,pjhd->pihd", dS, K)
        dk[rows] = scale * np.einsum("phij,pihd->pjhd", dS, Q)
    return dq, dk, dv


def fp8_e4m3_decode(codes) -> np.ndarray:
    """Values of 8-bit floating point codes in the E4M3 format of the OCP 8-bit floating
    point specification (the format of FP8 attention, Section 5.2): 1 sign, 4 exponent
    (bias 7), 3 mantissa bits; no infinities; exponent and mantissa all ones is NaN;
    exponent 0 is subnormal, (m/8) * 2**-6.  Largest finite value 448.  Returns fp64."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    val = np.where(e == 0, (m / 8.0) * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e - 7.0))
    val = np.where((c & 0x7F) == 0x7F, np.nan, val)
    return sign * val


def fp8_e4m3_encode(x) -> np.ndarray:
    """Nearest E4M3 code of each value, ties to the even code, magnitudes beyond 448
    saturating to 448 (the quantiser clamps before it rounds).  NaN maps to 0x7F."""
    x = np.asarray(x, dtype=np.float64)
    grid = fp8_e4m3_decode(np.arange(0x7F, dtype=np.uint8))          # 0 .. 448, increasing
    a = np.minimum(np.abs(x), 448.0)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 0, 0x7E)     # first code with value >= a
    lo = np.maximum(hi - 1, 0)
    d_hi, d_lo = grid[hi] - a, a - grid[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    code = np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)
    return np.where(np.isnan(x), np.uint8(0x7F), code).astype(np.uint8)


def fp8_tile_exponent(amax) -> np.ndarray:
    """Scale exponent of a tile of values that is to be stored in E4M3 (FP8 attention, Section
    5.2; the paper names no scaling rule, the reading taken is one power-of-two scale per tile,
    which the matrix hardware applies exactly): the largest integer e with
        amax * 2**e <= 448        (448 = largest finite E4M3 value)
    where amax is the largest magnitude in the tile.  e is limited to [-120, 120] (scales travel
    as 8-bit exponents), and an all-zero tile takes e = 0.  The tile is stored as the E4M3
    codes of x * 2**e and read back as decode(code) * 2**-e.  Returns int64."""
    a = np.abs(np.asarray(amax, dtype=np.float64))
    m, x = np.frexp(a)                       # a = m * 2**x with m in [0.5, 1);  448 = 0.875 * 2**9
    e = np.where(m <= 0.875, 9 - x, 8 - x)
    e = np.clip(e, -120, 120)
    return np.where(a == 0.0, 0, e).astype(np.int64)


def _segment_of(cu: np.ndarray, n: int):
    s = int(np.searchsorted(cu, n, side="right")) - 1
    while cu[s + 1] == cu[s]:          # skip empty segments that share a boundary
        s += 1
    return int(cu[s]), int(cu[s + 1])


def attn_fwd_rows(q, k, v, cu_seqlens, scale: float, head: int, rows):
    """out and lse for selected packed query rows of one head.

    The same definition as attn_fwd, evaluated only for the query tokens in
    `rows` (each against all keys of its own segment).  Used where the whole
    tensor is too large to compute on the CPU.  Returns out [len(rows), D] and
    lse [len(rows)].
    """
    total, _, D = q.shape
    cu = _check_cu(cu_seqlens, total)
    rows = np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.size, D))
    lse = np.zeros(rows.size)
    for a, b in sorted({_segment_of(cu, int(n)) for n in rows}):
        sel = np.nonzero((rows >= a) & (rows < b))[0]
        K = _as_f64(k[a:b, head, :])
        V = _as_f64(v[a:b, head, :])
        Q = _as_f64(q[rows[sel], head, :])
        P, L = _softmax_rows(scale * (Q @ K.T))
        out[sel] = P @ V
        lse[sel] = L
    return out, lse


def attn_bwd_rows(q, k, v, dout, cu_seqlens, scale: float, head: int, rows):
    """dQ for selected query rows of one head, and those rows' share of dK, dV.

    dQ_i depends on query row i alone, so it is complete.  dK_j and dV_j are
    sums over query rows i; the returned dk_part, dv_part hold the terms of
    those sums with i in `rows` (summing the parts over a partition of a
    segment's rows gives that segment's dK, dV).  Shapes: dq [len(rows), D],
    dk_part and dv_part [total, D] (zero outside the touched segments).
    """
    total, _, D = q.shape
    cu = _check_cu(cu_seqlens, total)
    rows = np.asarray(rows, dtype=np.int64)
    dq = np.zeros((rows.size, D))
    dk_part = np.zeros((total, D))
    dv_part = np.zeros((total, D))
    for a, b in sorted({_segment_of(cu, int(n)) for n in rows}):
        sel = np.nonzero((rows >= a) & (rows < b))[0]
        K = _as_f64(k[a:b, head, :])
        V = _as_f64(v[a:b, head, :])
        Q = _as_f64(q[rows[sel], head, :])
        dO = _as_f64(dout[rows[sel], head, :])
        P, _ = _softmax_rows(scale * (Q @ K.T))
        O = P @ V
        delta = (dO * O).sum(axis=1, keepdims=True)
        dP = dO @ V.T
        dS = P * (dP - delta)
        dq[sel] = scale * (dS @ K)
        dk_part[a:b] += scale * (dS.T @ Q)
        dv_part[a:b] += P.T @ dO
    return dq, dk_part, dv_part


def attn_bwd_cols(q, k, v, dout, cu_seqlens, scale: float, head: int, cols, row_chunk: int = 4096):
    """dK and dV for selected packed key/value rows of one head (all in one segment).

    dK_j and dV_j are sums over every query row i of the segment, and each term
    needs that row's softmax normaliser and Delta_i, so the forward definition
    is evaluated for all rows of the segment first (rows are independent; they
    are visited `row_chunk` at a time only to bound memory).  Then, for j in
    `cols`:  P_ij = exp(S_ij - LSE_i), dV_j = sum_i P_ij dO_i,
    dS_ij = P_ij (dO_i . V_j - Delta_i), dK_j = scale * sum_i dS_ij Q_i.
    Returns dk [len(cols), D], dv [len(cols), D].
    """
    total, _, D = q.shape
    cu = _check_cu(cu_seqlens, total)
    cols = np.asarray(cols, dtype=np.int64)
    a, b = _segment_of(cu, int(cols[0]))
    if np.any(cols < a) or np.any(cols >= b):
        raise ValueError("all columns must lie in one segment")
    K = _as_f64(k[a:b, head, :])
    V = _as_f64(v[a:b, head, :])
    Kc = _as_f64(k[cols, head, :])
    Vc = _as_f64(v[cols, head, :])
    dk = np.zeros((cols.size, D))
    dv = np.zeros((cols.size, D))
    for r0 in range(a, b, row_chunk):
        r1 = min(b, r0 + row_chunk)
        Q = _as_f64(q[r0:r1, head, :])
        dO = _as_f64(dout[r0:r1, head, :])
        P, L = _softmax_rows(scale * (Q @ K.T))
        delta = (dO * (P @ V)).sum(axis=1, keepdims=True)
        del P
        Pc = np.exp(scale * (Q @ Kc.T) - L[:, None])
        dv += Pc.T @ dO
        dS = Pc * (dO @ Vc.T - delta)
        dk += scale * (dS.T @ Q)
    return dk, dv
