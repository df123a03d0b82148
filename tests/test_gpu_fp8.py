"""GPU parity of the FP8 (E4M3) attention forward with per-tile power-of-two scales: the packing
pass bit for bit against the oracle's quantiser and scale rule, and the attention output against
the fp64 oracle run on the SAME quantised operands (so operand quantisation is not charged).

Tolerance of `out` on the same operands, derived from the arithmetic: the probabilities are
rounded to E4M3 (3 mantissa bits) before the second product, a relative error uniform in
+-2^-4 per term, RMS 2^-4/sqrt(3) = 3.6%.  out_i = sum_j p_ij v_j with independent errors e_ij has
error sum_j e_ij p_ij v_j, RMS 3.6% * sqrt(sum_j p_ij^2 v_j^2); for the zero-mean synthetic values
|out_i| itself is a random walk of the same terms, about sqrt(sum_j p_ij^2 v_j^2), so the relative
RMS error is 3.6% however many keys there are (it does not average out; real activations with a
mean component fare better).  fp32 accumulation and the bf16 rounding of out add 0.2%.  Bound:
5e-2 on the tensor, and 3x that on every (token, head) row.  lse never sees P: 1e-3 as for bf16."""
import numpy as np
import pytest

from oracle import vfm_oracle as orc
from paper_2503_12964_amd import workloads as W
from tests import parity_utils as U
from tests.test_gpu_parity import SMALL, _binding, _custom

pytestmark = pytest.mark.gpu

TOL_FP8_OUT_RELRMS = 5e-2
LOG2E = 1.4426950408889634


def _pre(wl):
    """What q is multiplied by before it is quantised (softmax scale in log2 units), formed in
    fp32 exactly as the library forms it."""
    return np.float32(np.float32(wl.scale) * np.float32(LOG2E))


def _unit_starts(cu):
    """(first key, valid keys) of every 64-key unit, clip by clip in packed order."""
    units = []
    for a, b in zip(cu[:-1], cu[1:]):
        units += [(int(k0), int(min(64, b - k0))) for k0 in range(int(a), int(b), 64)]
    return units


def _expected(wl, inp):
    """Oracle side of the packing pass: tile exponents by the oracle's rule, codes by its encoder.
    The products are formed in fp32 as the kernel forms them; scaling by 2^e is exact."""
    x = {n: W.bf16_bits_to_f32(inp[n]) for n in ("q", "k", "v")}
    qs = x["q"] * _pre(wl)                                             # fp32 product
    e_q = orc.fp8_tile_exponent(np.abs(qs).max(axis=2))                # [total, heads]
    want = {"q": orc.fp8_e4m3_encode(qs.astype(np.float64) * 2.0 ** e_q[:, :, None]), "e_q": e_q}
    units = _unit_starts(wl.cu_seqlens)
    for n in ("k", "v"):
        e = np.zeros((len(units), wl.n_heads), dtype=np.int64)
        codes = np.zeros(x[n].shape, dtype=np.uint8)
        for u, (k0, m) in enumerate(units):
            tile = x[n][k0:k0 + m].astype(np.float64)                  # [m, heads, D]
            e[u] = orc.fp8_tile_exponent(np.abs(tile).max(axis=(0, 2)))
            codes[k0:k0 + m] = orc.fp8_e4m3_encode(tile * 2.0 ** e[u][None, :, None])
        want[n], want["e_" + n] = codes, e
    return want


def _dequantised(wl, want):
    """The values the tiles read back as (q without the factor it carried)."""
    units = _unit_starts(wl.cu_seqlens)
    deq = {"q": orc.fp8_e4m3_decode(want["q"]) * 2.0 ** -want["e_q"][:, :, None] / float(_pre(wl))}
    for n in ("k", "v"):
        d = orc.fp8_e4m3_decode(want[n])
        for u, (k0, m) in enumerate(units):
            d[k0:k0 + m] *= 2.0 ** -want["e_" + n][u][None, :, None]
        deq[n] = d
    return deq


def _unpack(cu, heads, hd, q8, k8, vT8, scales):
    """Undo the packed layout (as include/vfm.h states it) -> code arrays [total, heads, hd] and
    the tile exponents."""
    total = int(cu[-1])
    lens = np.diff(cu)
    units = [(n + 63) // 64 for n in lens]
    n_units = int(sum(units))
    q = q8.reshape(heads, total, hd).transpose(1, 0, 2)
    e_q = 127 - scales[:heads * total].reshape(heads, total).T.astype(np.int64)
    words = scales[(heads * total + 255) // 256 * 256:][:heads * n_units * 4].reshape(heads, n_units, 4)
    e_k = 127 - words[:, :, 0].T.astype(np.int64)
    e_v = 127 - words[:, :, 1].T.astype(np.int64)
    tail_ok = bool(np.all(words[:, :, 2:] == 127))
    kk = k8.reshape(heads, n_units, 64, hd // 16, 16)
    vv = vT8.reshape(heads, n_units, hd, 4, 16)
    k = np.zeros((total, heads, hd), np.uint8)
    v = np.zeros((total, heads, hd), np.uint8)
    pad_ok = True
    r = np.arange(64)
    kswz = ((r >> 1) & 7) if hd == 128 else ((r >> 2) & 3)
    d = np.arange(hd)
    vswz = (d >> 2) & 3
    b = np.arange(64)                               # logical byte of a V^T row -> key of the unit
    g, j = b // 32, b % 32
    key_of_byte = 32 * (j // 16) + 8 * ((j % 16) // 4) + 4 * g + j % 4
    u0 = 0
    for s, n in enumerate(lens):
        for u in range(units[s]):
            a = int(cu[s]) + 64 * u
            m = min(64, int(cu[s + 1]) - a)
            ku = kk[:, u0 + u]                      # [heads, 64, chunks, 16]
            logical = np.empty_like(ku)
            for c in range(hd // 16):
                logical[:, r, c] = ku[:, r, c ^ kswz]
            rows = logical.reshape(heads, 64, hd)
            k[a:a + m] = rows[:, :m].transpose(1, 0, 2)
            pad_ok &= not np.any(rows[:, m:])
            vu = vv[:, u0 + u]                      # [heads, hd, 4, 16]
            vlog = np.empty_like(vu)
            for c in range(4):
                vlog[:, d, c] = vu[:, d, c ^ vswz]
            vrow = vlog.reshape(heads, hd, 64)      # [heads, d, logical byte]
            by_key = np.empty_like(vrow)
            by_key[:, :, key_of_byte] = vrow
            v[a:a + m] = by_key[:, :, :m].transpose(2, 0, 1)
            pad_ok &= not np.any(by_key[:, :, m:])
        u0 += units[s]
    return {"q": q, "k": k, "v": v, "e_q": e_q, "e_k": e_k, "e_v": e_v}, pad_ok and tail_ok


def _pack(b, wl, inp=None):
    inp = W.make_inputs(wl, tensors=("q", "k", "v")) if inp is None else inp
    dev = {n: U.to_device(inp[n]) for n in ("q", "k", "v")}
    return inp, b.vfm_fp8_pack(dev["q"], dev["k"], dev["v"], wl.cu_seqlens, wl.scale)


def _check_pack_and_attention(b, wl, inp, lse_tol=U.TOL_LSE_MAXABS):
    inp, (q8, k8, vT8, scales) = _pack(b, wl, inp)
    nq, nk, nv, ns = b.vfm_fp8_pack_sizes(wl.cu_seqlens, wl.n_heads, wl.head_dim)
    got, pad_ok = _unpack(wl.cu_seqlens, wl.n_heads, wl.head_dim, q8.cpu().numpy()[:nq], k8.cpu().numpy()[:nk],
                          vT8.cpu().numpy()[:nv], scales.cpu().numpy()[:ns])
    assert pad_ok, "padding keys of a unit must be zero, spare scale bytes 127"
    want = _expected(wl, inp)
    for key in ("e_q", "e_k", "e_v", "q", "k", "v"):            # exponents and codes bit for bit
        assert np.array_equal(got[key], want[key]), key
    out, lse = b.vfm_attn_fwd_fp8(q8, k8, vT8, scales, wl.cu_seqlens, wl.n_heads, wl.head_dim)
    deq = _dequantised(wl, want)
    o_ref, l_ref = orc.attn_fwd(deq["q"], deq["k"], deq["v"], wl.cu_seqlens, wl.scale)
    o = U.to_f64(out)
    assert np.all(np.isfinite(o))
    assert U.rel_rms(o, o_ref) <= TOL_FP8_OUT_RELRMS
    U.assert_rows_close("out", o, o_ref, TOL_FP8_OUT_RELRMS)
    assert U.max_abs(U.to_f64(lse), l_ref) <= lse_tol
    return o, deq


# clips of 3, 4, 6, 7, 8 and 10 key units (64 keys each): every way the unit loop, which is
# unrolled four times after its first unit, can end; the last two span more than one query tile
FP8_CASES = dict(SMALL)
FP8_CASES["units_mix"] = _custom("units_mix", [(1, 10, 13), (1, 16, 16), (1, 15, 22), (1, 20, 20), (2, 16, 16),
                                               (1, 23, 27)], 2, 128, (32, 48, 48), 21)


@pytest.mark.parametrize("name", ["ragged128", "ragged64", "units_mix"])
def test_pack_is_bit_exact_and_attention_matches_oracle(name):
    wl = FP8_CASES[name]
    b = _binding()
    inp = W.make_inputs(wl, tensors=("q", "k", "v"))
    o, _ = _check_pack_and_attention(b, wl, inp)
    # and it is still attention on the original tensors, to operand-quantisation accuracy
    f64 = {n: U.bits_to_f64(inp[n]) for n in ("q", "k", "v")}
    o_true, _ = orc.attn_fwd(f64["q"], f64["k"], f64["v"], wl.cu_seqlens, wl.scale)
    assert U.rel_rms(o, o_true) <= 2 * TOL_FP8_OUT_RELRMS


def test_tiles_of_very_different_magnitude_keep_their_precision():
    # Clips whose k is 2^-5 to 2^5 and whose v is 2^-12 to 2^10 times unit variance (q carries the
    # inverse of the k factor, so the scores stay ordinary).  With a scale per tile every tile uses
    # E4M3's top binade, and every clip's output is as accurate as for unit-variance data.  One
    # scale per tensor, sized for the tensor's maximum, pushes the small clips into the
    # subnormals or to zero: evaluated with the oracle alone, such clips come out wrong.
    wl = FP8_CASES["units_mix"]
    b = _binding()
    inp = W.make_inputs(wl, tensors=("q", "k", "v"))
    f32 = {n: W.bf16_bits_to_f32(inp[n]) for n in inp}
    cu = wl.cu_seqlens
    for c, (ka, vb) in enumerate(zip((-5, 3, 0, 5, -2, 4), (-12, 10, -3, 4, -9, 0))):
        a, e = int(cu[c]), int(cu[c + 1])
        f32["k"][a:e] *= np.float32(2.0 ** ka)
        f32["q"][a:e] *= np.float32(2.0 ** -ka)
        f32["v"][a:e] *= np.float32(2.0 ** vb)
    inp = {n: W.f32_to_bf16_bits(x) for n, x in f32.items()}
    o, deq = _check_pack_and_attention(b, wl, inp)
    f64 = {n: U.bits_to_f64(inp[n]) for n in inp}
    o_true, _ = orc.attn_fwd(f64["q"], f64["k"], f64["v"], cu, wl.scale)
    pre = float(_pre(wl))
    one = {}
    for n in ("q", "k", "v"):
        x = f64[n] * (pre if n == "q" else 1.0)
        e = int(orc.fp8_tile_exponent(np.abs(x).max()))
        one[n] = orc.fp8_e4m3_decode(orc.fp8_e4m3_encode(x * 2.0 ** e)) * 2.0 ** -e / (pre if n == "q" else 1.0)
    o_one, _ = orc.attn_fwd(one["q"], one["k"], one["v"], cu, wl.scale)
    per_tile = [U.rel_rms(o[a:e], o_true[a:e]) for a, e in zip(cu[:-1], cu[1:])]
    per_tensor = [U.rel_rms(o_one[a:e], o_true[a:e]) for a, e in zip(cu[:-1], cu[1:])]
    assert max(per_tile) <= 2 * TOL_FP8_OUT_RELRMS, per_tile
    assert max(per_tensor) > 0.5, per_tensor


def test_growing_scores_move_the_reference():
    wl = SMALL["ragged128"]
    b = _binding()
    inp = W.make_inputs(wl, tensors=("q", "k", "v"))
    ramp = np.linspace(1.0, 12.0, wl.total_tokens, dtype=np.float32)
    inp["k"] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(inp["k"]) * ramp[:, None, None])
    _check_pack_and_attention(b, wl, inp, lse_tol=2e-3)


def test_more_clips_than_a_table_holds():
    rng = np.random.default_rng(42)
    grids = tuple((1, 1, int(n)) for n in rng.integers(0, 150, size=300))
    wl = W.Workload("fp8_300", grids, 2, 128, (32, 48, 48), seed=43)
    _check_pack_and_attention(_binding(), wl, W.make_inputs(wl, tensors=("q", "k", "v")))


def test_headline_shape_sampled_rows_on_full_heads():
    """56,320 tokens, 32 heads: the packing pass on three whole heads bit for bit, and sampled
    query rows of those heads (clip ends, tile boundaries, random rows) against the oracle on the
    quantised operands, with the per-row bound."""
    wl = W.WORKLOADS["C4"]
    b = _binding()
    inp, (q8, k8, vT8, scales) = _pack(b, wl)
    out, lse = b.vfm_attn_fwd_fp8(q8, k8, vT8, scales, wl.cu_seqlens, wl.n_heads, wl.head_dim)
    nq, nk, nv, ns = b.vfm_fp8_pack_sizes(wl.cu_seqlens, wl.n_heads, wl.head_dim)
    total, H, D = wl.total_tokens, wl.n_heads, wl.head_dim
    n_units = total // 64
    sc = scales.cpu().numpy()[:ns]
    words = sc[(H * total + 255) // 256 * 256:].reshape(H, n_units, 4)
    rows = np.unique(np.concatenate([[0, 255, 256, 56319], np.random.default_rng(9).integers(0, 56320, 60)]))
    err = ref = 0.0
    for h in (0, 13, 31):
        one = W.Workload("c4_head", wl.grids, 1, D, wl.rope_dims, wl.seed)
        sub = {n: np.ascontiguousarray(inp[n][:, h:h + 1]) for n in ("q", "k", "v")}
        want = _expected(one, sub)
        assert np.array_equal(127 - sc[h * total:(h + 1) * total].astype(np.int64), want["e_q"][:, 0])
        assert np.array_equal(127 - words[h, :, 0].astype(np.int64), want["e_k"][:, 0])
        assert np.array_equal(127 - words[h, :, 1].astype(np.int64), want["e_v"][:, 0])
        assert np.array_equal(q8[h * total * D:(h + 1) * total * D].cpu().numpy().reshape(total, D), want["q"][:, 0])
        deq = _dequantised(one, want)
        o_ref, l_ref = orc.attn_fwd_rows(deq["q"], deq["k"], deq["v"], wl.cu_seqlens, wl.scale, 0, rows)
        o = U.to_f64(out[rows, h, :])
        U.assert_rows_close("out", o, o_ref, TOL_FP8_OUT_RELRMS)
        err += np.sum((o - o_ref) ** 2)
        ref += np.sum(o_ref ** 2)
        assert U.max_abs(U.to_f64(lse[h, rows]), l_ref) <= U.TOL_LSE_MAXABS
    assert np.sqrt(err / ref) <= TOL_FP8_OUT_RELRMS
