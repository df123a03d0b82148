"""Planted mistakes for the oracle (CPU only, test infrastructure).

Each entry rewrites one expression of oracle/vfm_oracle.py into a plausible mistake: a dropped
term or factor, a wrong sign, a wrong index or axis, a transposed operand.  `install(name)`
compiles the rewritten source into a throw-away module and replaces the functions of the
imported oracle module with it, so that the pin tests (which reach the oracle through that
module's attributes) run against the mistaken oracle.  tests/test_oracle_mutations.py checks
that the pins reject every one of them.  Nothing here touches the GPU path.
"""
from __future__ import annotations

import os
import types

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_SRC = os.path.join(ROOT, "oracle", "vfm_oracle.py")

# name -> (text to find, replacement, which occurrence of the text (0-based))
MUTANTS = {
    # ---- token -> (t, h, w)
    "coords_t_fastest": ("pos[a:b, 0] = r // (H * W)", "pos[a:b, 0] = r % T", 0),
    "coords_h_by_wrong_extent": ("pos[a:b, 1] = (r // W) % H", "pos[a:b, 1] = (r // H) % W", 0),
    "coords_w_by_wrong_extent": ("pos[a:b, 2] = r % W", "pos[a:b, 2] = r % H", 0),
    # ---- 3D RoPE
    "rope_exponent_without_2": ("(-2.0 * i / d_a)", "(-1.0 * i / d_a)", 0),
    "rope_exponent_over_head_dim": ("(-2.0 * i / d_a)", "(-2.0 * i / D)", 0),
    "rope_one_sign_wrong": ("= x0 * c - x1 * s", "= x0 * c + x1 * s", 0),
    "rope_direction_reversed": ("phi = pos[:, axis]", "phi = -pos[:, axis]", 0),
    "rope_slice_offset_stuck": ("        start += d_a\n", "        start += 0\n", 0),
    "rope_inverse_ignored": ("            phi = -phi\n", "            phi = +phi\n", 0),
    "rope_every_axis_uses_t": ("phi = pos[:, axis]", "phi = pos[:, 0]", 0),
    "rope_theta_inverted": ("freq = float(theta) ** (", "freq = float(theta) ** -(", 0),
    # ---- per-head normalisation
    "norm_sum_instead_of_mean": ("np.sqrt(np.mean(x * x, axis=2, keepdims=True)", "np.sqrt(np.sum(x * x, axis=2, keepdims=True)", 0),
    "norm_eps_outside_sqrt": ("np.sqrt(np.mean(x * x, axis=2, keepdims=True) + float(eps))",
                              "(np.sqrt(np.mean(x * x, axis=2, keepdims=True)) + float(eps))", 0),
    "norm_gain_dropped": ("z = x * _rstd(x, eps) * g[None, None, :]", "z = x * _rstd(x, eps)", 0),
    "norm_bwd_sum_instead_of_mean": ("np.mean(dn * n, axis=2, keepdims=True)", "np.sum(dn * n, axis=2, keepdims=True)", 0),
    "norm_bwd_projection_dropped": ("dx = r * (dn - n * np.mean(dn * n, axis=2, keepdims=True))", "dx = r * dn", 0),
    "norm_bwd_dgain_from_x": ("dgain = np.sum(dz * n, axis=(0, 1))", "dgain = np.sum(dz * x, axis=(0, 1))", 0),
    "norm_bwd_rotation_not_transposed": ("dims, theta, inverse=True)", "dims, theta, inverse=False)", 0),
    # ---- softmax attention, forward
    "lse_without_max": ("return E / l, (m + np.log(l))[:, 0]", "return E / l, (np.log(l))[:, 0]", 0),
    "softmax_not_normalised": ("return E / l, (m", "return E, (m", 0),
    "fwd_scale_dropped": ("S = scale * (q[a:b, h, :] @ k[a:b, h, :].T)", "S = (q[a:b, h, :] @ k[a:b, h, :].T)", 0),
    "fwd_p_transposed": ("out[a:b, h, :] = P @ v[a:b, h, :]", "out[a:b, h, :] = P.T @ v[a:b, h, :]", 0),
    "fwd_q_and_k_swapped": ("S = scale * (q[a:b, h, :] @ k[a:b, h, :].T)", "S = scale * (k[a:b, h, :] @ q[a:b, h, :].T)", 0),
    # ---- softmax attention, backward
    "bwd_delta_dropped": ("dS = P * (dP - delta)\n            dq[a:b", "dS = P * dP\n            dq[a:b", 0),
    "bwd_delta_sign": ("dS = P * (dP - delta)\n            dq[a:b", "dS = P * (dP + delta)\n            dq[a:b", 0),
    "bwd_delta_from_v": ("delta = (dO * O).sum(axis=1, keepdims=True)\n            dv[a:b", "delta = (dO * V).sum(axis=1, keepdims=True)\n            dv[a:b", 0),
    "bwd_given_out_ignored": ("O = P @ V if given is None else given[a:b, h, :]", "O = P @ V", 0),
    "bwd_given_out_of_head_zero": ("O = P @ V if given is None else given[a:b, h, :]",
                                   "O = P @ V if given is None else given[a:b, 0, :]", 0),
    "bwd_dq_scale_dropped": ("dq[a:b, h, :] = scale * (dS @ K)", "dq[a:b, h, :] = (dS @ K)", 0),
    "bwd_dk_not_transposed": ("dk[a:b, h, :] = scale * (dS.T @ Q)", "dk[a:b, h, :] = scale * (dS @ Q)", 0),
    "bwd_dq_transposed": ("dq[a:b, h, :] = scale * (dS @ K)", "dq[a:b, h, :] = scale * (dS.T @ K)", 0),
    "bwd_dv_not_transposed": ("dv[a:b, h, :] = P.T @ dO", "dv[a:b, h, :] = P @ dO", 0),
    "bwd_dp_from_k": ("dP = dO @ V.T\n            dS = P * (dP - delta)\n            dq[a:b", "dP = dO @ K.T\n            dS = P * (dP - delta)\n            dq[a:b", 0),
    "bwd_segment_starts_at_zero": ("a, b = int(cu[s]), int(cu[s + 1])", "a, b = 0, int(cu[s + 1])", 2),
    "fwd_segment_starts_at_zero": ("a, b = int(cu[s]), int(cu[s + 1])", "a, b = 0, int(cu[s + 1])", 1),
    # ---- cross-attention
    "x_bwd_delta_dropped": ("dS = P * (dO @ V.T - delta)", "dS = P * (dO @ V.T)", 0),
    "x_bwd_dk_scale_dropped": ("dk[c:d, h, :] = scale * (dS.T @ Q)", "dk[c:d, h, :] = (dS.T @ Q)", 0),
    "x_bwd_dq_from_v": ("dq[a:b, h, :] = scale * (dS @ K)\n            dk[c:d", "dq[a:b, h, :] = scale * (dS @ V)\n            dk[c:d", 0),
    "x_fwd_keys_of_first_sequence": ("P, L = _softmax_rows(scale * (q[a:b, h, :] @ k[c:d, h, :].T))\n            out[a:b, h, :] = P @ v[c:d, h, :]",
                                     "c, d = int(ck[0]), int(ck[1])\n            P, L = _softmax_rows(scale * (q[a:b, h, :] @ k[c:d, h, :].T))\n            out[a:b, h, :] = P @ v[c:d, h, :]", 0),
    # ---- temporal attention
    "t_rows_t_fastest": ("np.arange(T)[None, :] * (H * W) + np.arange(H * W)[:, None]", "np.arange(T)[None, :] + np.arange(H * W)[:, None] * T", 0),
    "t_fwd_p_transposed": ('out[rows] = np.einsum("phij,pjhd->pihd", P, V)', 'out[rows] = np.einsum("phji,pjhd->pihd", P, V)', 0),
    "t_fwd_softmax_over_queries": ("S -= S.max(axis=3, keepdims=True)\n        P = np.exp(S)\n        P /= P.sum(axis=3, keepdims=True)\n        out[rows]",
                                   "S -= S.max(axis=2, keepdims=True)\n        P = np.exp(S)\n        P /= P.sum(axis=2, keepdims=True)\n        out[rows]", 0),
    "t_bwd_delta_dropped": ("dS = P * (dP - delta)\n        dv[rows]", "dS = P * dP\n        dv[rows]", 0),
    "t_bwd_dk_indices": ('dk[rows] = scale * np.einsum("phij,pihd->pjhd", dS, Q)', 'dk[rows] = scale * np.einsum("phji,pihd->pjhd", dS, Q)', 0),
    "t_bwd_dq_scale_dropped": ('dq[rows] = scale * np.einsum("phij,pjhd->pihd", dS, K)', 'dq[rows] = np.einsum("phij,pjhd->pihd", dS, K)', 0),
    # ---- E4M3 codes
    "fp8_bias_8": ("2.0 ** (e - 7.0)", "2.0 ** (e - 8.0)", 0),
    "fp8_subnormal_scale": ("(m / 8.0) * 2.0 ** -6", "(m / 8.0) * 2.0 ** -7", 0),
    "fp8_ties_to_odd": ("(lo % 2 == 0)", "(lo % 2 == 1)", 0),
    "fp8_truncates": ("pick_lo = (d_lo < d_hi) |", "pick_lo = (d_lo >= 0) |", 0),
    "fp8_sign_lost": ("code = np.where(np.signbit(x), code | 0x80, code)", "code = np.where(np.signbit(x), code, code)", 0),
    "fp8_tile_exponent_off_by_one": ("e = np.where(m <= 0.875, 9 - x, 8 - x)", "e = np.where(m <= 0.875, 8 - x, 7 - x)", 0),
    "fp8_tile_exponent_boundary": ("e = np.where(m <= 0.875, 9 - x, 8 - x)", "e = np.where(m < 0.875, 9 - x, 8 - x)", 0),
    "fp8_tile_exponent_to_256": ("e = np.where(m <= 0.875, 9 - x, 8 - x)", "e = np.where(m <= 0.5, 9 - x, 8 - x)", 0),
    # ---- helpers for sampled rows and columns of large cases
    "rows_dq_scale_dropped": ("dq[sel] = scale * (dS @ K)", "dq[sel] = (dS @ K)", 0),
    "rows_delta_dropped": ("dS = P * (dP - delta)\n        dq[sel]", "dS = P * dP\n        dq[sel]", 0),
    "rows_fwd_keys_of_whole_tensor": ("K = _as_f64(k[a:b, head, :])\n        V = _as_f64(v[a:b, head, :])\n        Q = _as_f64(q[rows[sel], head, :])\n        P, L",
                                      "K = _as_f64(k[:, head, :])\n        V = _as_f64(v[:, head, :])\n        Q = _as_f64(q[rows[sel], head, :])\n        P, L", 0),
    "cols_normaliser_dropped": ("Pc = np.exp(scale * (Q @ Kc.T) - L[:, None])", "Pc = np.exp(scale * (Q @ Kc.T))", 0),
}


def mutated_source(name: str) -> str:
    old, new, which = MUTANTS[name]
    src = open(ORACLE_SRC).read()
    at = -1
    for _ in range(which + 1):
        at = src.find(old, at + 1)
        if at < 0:
            raise KeyError(f"mutant {name}: text not found in the oracle: {old!r}")
    return src[:at] + new + src[at + len(old):]


def install(name: str) -> None:
    """Replace the functions of the imported oracle module by the mistaken ones."""
    from oracle import vfm_oracle as orc
    mod = types.ModuleType("vfm_oracle_mutant_" + name)
    exec(compile(mutated_source(name), ORACLE_SRC + "<" + name + ">", "exec"), mod.__dict__)
    for key, val in mod.__dict__.items():
        if callable(val) and getattr(val, "__module__", None) == mod.__name__:
            setattr(orc, key, val)
