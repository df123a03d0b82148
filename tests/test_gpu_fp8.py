"""GPU parity of the FP8 (E4M3) attention forward: the packing pass bit for bit against the
oracle's quantiser, and the attention output against the fp64 oracle run on the SAME quantised
operands (so operand quantisation is not charged; what remains is the E4M3 rounding of the
probabilities, 3 mantissa bits: relative error uniform in +-2^-4 per term, RMS 2^-4/sqrt(3) = 3.6%,
which for zero-mean synthetic values does not average out against |out|)."""
import numpy as np
import pytest

from oracle import vfm_oracle as orc
from paper_2503_12964_amd import workloads as W
from tests import parity_utils as U
from tests.test_gpu_parity import SMALL, _binding, _custom

pytestmark = pytest.mark.gpu

TOL_FP8_OUT_RELRMS = 5e-2
LOG2E = 1.4426950408889634
K_SCALE, V_SCALE = 1.0, 16.0       # powers of two; N(0,1) draws stay far below 448


def _mults(wl):
    """Multipliers the pack applies to q, k, v (q carries the softmax scale in log2 units); the q
    multiplier is formed in fp32 exactly as the library forms it."""
    qm = np.float32(np.float32(wl.scale) * np.float32(LOG2E)) / np.float32(K_SCALE)
    return (float(qm), K_SCALE, V_SCALE)


def _unpack(cu, heads, hd, q8, k8, vT8):
    """Undo the packed layout (as include/vfm.h states it) -> code arrays [total, heads, hd]."""
    total = int(cu[-1])
    lens = np.diff(cu)
    units = [(n + 63) // 64 for n in lens]
    n_units = int(sum(units))
    q = q8.reshape(heads, total, hd).transpose(1, 0, 2)
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
    return q, k, v, pad_ok


def _pack(b, wl):
    inp = W.make_inputs(wl, tensors=("q", "k", "v"))
    dev = {n: U.to_device(inp[n]) for n in ("q", "k", "v")}
    q8, k8, vT8 = b.vfm_fp8_pack(dev["q"], dev["k"], dev["v"], wl.cu_seqlens, wl.scale, K_SCALE, V_SCALE)
    return inp, (q8, k8, vT8)


# clips of 3, 4, 6, 7, 8 and 10 key units (64 keys each): every way the unit loop, which is
# unrolled four times after its first unit, can end; the last two span more than one query tile
FP8_CASES = dict(SMALL)
FP8_CASES["units_mix"] = _custom("units_mix", [(1, 10, 13), (1, 16, 16), (1, 15, 22), (1, 20, 20), (2, 16, 16),
                                               (1, 23, 27)], 2, 128, (32, 48, 48), 21)


@pytest.mark.parametrize("name", ["ragged128", "ragged64", "units_mix"])
def test_pack_is_bit_exact_and_attention_matches_oracle(name):
    wl = FP8_CASES[name]
    b = _binding()
    inp, (q8, k8, vT8) = _pack(b, wl)
    nq, nk, nv = b.vfm_fp8_pack_sizes(wl.cu_seqlens, wl.n_heads, wl.head_dim)
    codes = _unpack(wl.cu_seqlens, wl.n_heads, wl.head_dim, q8.cpu().numpy()[:nq], k8.cpu().numpy()[:nk],
                    vT8.cpu().numpy()[:nv])
    assert codes[3], "padding keys of a unit must be zero"
    deq = {}
    for nm, got, sc in zip(("q", "k", "v"), codes[:3], _mults(wl)):
        want = orc.fp8_e4m3_encode(W.bf16_bits_to_f32(inp[nm]) * np.float32(sc))   # fp32 product, as the kernel
        assert np.array_equal(got, want), nm
        deq[nm] = orc.fp8_e4m3_decode(got) / sc
    out, lse = b.vfm_attn_fwd_fp8(q8, k8, vT8, wl.cu_seqlens, wl.n_heads, wl.head_dim, V_SCALE)
    o_ref, l_ref = orc.attn_fwd(deq["q"], deq["k"], deq["v"], wl.cu_seqlens, wl.scale)
    o = U.to_f64(out)
    assert np.all(np.isfinite(o))
    assert U.rel_rms(o, o_ref) <= TOL_FP8_OUT_RELRMS
    assert U.max_abs(U.to_f64(lse), l_ref) <= U.TOL_LSE_MAXABS
    # and it is still attention on the original tensors, to operand-quantisation accuracy
    f64 = {n: U.bits_to_f64(inp[n]) for n in ("q", "k", "v")}
    o_true, _ = orc.attn_fwd(f64["q"], f64["k"], f64["v"], wl.cu_seqlens, wl.scale)
    assert U.rel_rms(o, o_true) <= 2 * TOL_FP8_OUT_RELRMS


def test_growing_scores_move_the_reference():
    import torch
    wl = SMALL["ragged128"]
    b = _binding()
    inp = W.make_inputs(wl, tensors=("q", "k", "v"))
    dev = {n: U.to_device(inp[n]) for n in ("q", "k", "v")}
    ramp = torch.linspace(1.0, 12.0, wl.total_tokens, device="cuda")
    dev["k"] = (dev["k"].float() * ramp[:, None, None]).to(torch.bfloat16)
    scales = _mults(wl)
    q8, k8, vT8 = b.vfm_fp8_pack(dev["q"], dev["k"], dev["v"], wl.cu_seqlens, wl.scale, K_SCALE, V_SCALE)
    out, lse = b.vfm_attn_fwd_fp8(q8, k8, vT8, wl.cu_seqlens, wl.n_heads, wl.head_dim, V_SCALE)
    deq = {}
    for nm, sc in zip(("q", "k", "v"), scales):
        x32 = dev[nm].float().cpu().numpy() * np.float32(sc)
        deq[nm] = orc.fp8_e4m3_decode(orc.fp8_e4m3_encode(x32)) / sc
    o_ref, l_ref = orc.attn_fwd(deq["q"], deq["k"], deq["v"], wl.cu_seqlens, wl.scale)
    o = U.to_f64(out)
    assert np.all(np.isfinite(o))
    assert U.rel_rms(o, o_ref) <= TOL_FP8_OUT_RELRMS
    assert U.max_abs(U.to_f64(lse), l_ref) <= 2e-3


def test_headline_shape_sampled_rows():
    """56,320 tokens, 32 heads: sampled query rows of four heads against the oracle on the
    quantised operands."""
    wl = W.WORKLOADS["C4"]
    b = _binding()
    inp, (q8, k8, vT8) = _pack(b, wl)
    out, lse = b.vfm_attn_fwd_fp8(q8, k8, vT8, wl.cu_seqlens, wl.n_heads, wl.head_dim, V_SCALE)
    rows = np.unique(np.concatenate([[0, 255, 256, 56319], np.random.default_rng(9).integers(0, 56320, 24)]))
    err = ref = 0.0
    for h in (0, 13, 31):
        deq = {}
        for nm, sc in zip(("q", "k", "v"), _mults(wl)):
            x32 = W.bf16_bits_to_f32(inp[nm][:, h:h + 1]) * np.float32(sc)
            deq[nm] = orc.fp8_e4m3_decode(orc.fp8_e4m3_encode(x32)) / sc
        o_ref, l_ref = orc.attn_fwd_rows(deq["q"], deq["k"], deq["v"], wl.cu_seqlens, wl.scale, 0, rows)
        o = U.to_f64(out[rows, h, :])
        err += np.sum((o - o_ref) ** 2)
        ref += np.sum(o_ref ** 2)
        assert U.max_abs(U.to_f64(lse[h, rows]), l_ref) <= U.TOL_LSE_MAXABS
    assert np.sqrt(err / ref) <= TOL_FP8_OUT_RELRMS
