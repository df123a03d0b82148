"""GPU parity of temporal attention (one sequence per pixel across a clip's frames) against the
fp64 oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import vfm_oracle as orc
from paper_2503_12964_amd import workloads as W
from tests import parity_utils as U

pytestmark = pytest.mark.gpu


def _binding():
    from paper_2503_12964_amd import binding
    binding.load_library()
    return binding


CASES = {
    # frame counts 1, 2, 7, 16 and an empty clip; pixel counts that are not multiples of the 4 waves
    "t128": W.Workload("t128", ((16, 3, 5), (1, 2, 3), (0, 1, 1), (7, 1, 1), (2, 5, 5)), 3, 128, (32, 48, 48), seed=31),
    "t64": W.Workload("t64", ((5, 3, 3), (16, 1, 2), (3, 4, 1)), 2, 64, (16, 24, 24), seed=32),
    # more than 16 frames (the 32-row tile): 17, 24, 32 frames mixed with short clips, an empty one and
    # a single-frame one in the same call
    "t128_long": W.Workload("t128_long", ((17, 2, 3), (4, 3, 3), (32, 1, 5), (0, 1, 1), (24, 2, 2), (1, 3, 1)), 3, 128,
                            (32, 48, 48), seed=33),
    "t64_long": W.Workload("t64_long", ((32, 3, 1), (9, 2, 2), (20, 1, 1)), 2, 64, (16, 24, 24), seed=34),
}


def _check(wl, gpu, dev, heads=None):
    out, dq, dk, dv = gpu
    hs = slice(None) if heads is None else list(heads)
    host = {n: U.to_f64(t[:, hs, :]) for n, t in dev.items()}
    o_ref = orc.temporal_attn_fwd(host["q"], host["k"], host["v"], wl.thw, wl.cu_seqlens, wl.scale)
    g_ref = orc.temporal_attn_bwd(host["q"], host["k"], host["v"], host["dout"], wl.thw, wl.cu_seqlens, wl.scale)
    o = U.to_f64(out[:, hs, :])
    assert np.all(np.isfinite(o))
    # at most 32 keys: outputs are O(|v|), so the absolute bound is taken relative to max(1, |ref|)
    assert np.max(np.abs(o - o_ref) / np.maximum(1.0, np.abs(o_ref))) <= U.TOL_OUT_MAXABS
    assert U.rel_rms(o, o_ref) <= U.TOL_OUT_RELRMS
    U.assert_rows_close("out", o, o_ref, U.TOL_OUT_RELRMS)
    for nm, g, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), g_ref):
        got = U.to_f64(g[:, hs, :])
        assert np.all(np.isfinite(got))
        r = U.rel_rms(got, ref)
        assert r <= U.TOL_GRAD_RELRMS, (nm, r)
        U.assert_rows_close(nm, got, ref, U.TOL_GRAD_RELRMS)       # every (token, head) row


def _run(b, wl):
    inp = W.make_inputs(wl)
    dev = {n: U.to_device(inp[n]) for n in ("q", "k", "v", "dout")}
    out = b.vfm_tattn_fwd(dev["q"], dev["k"], dev["v"], wl.thw, wl.cu_seqlens, wl.scale)
    dq, dk, dv = b.vfm_tattn_bwd(dev["q"], dev["k"], dev["v"], dev["dout"], wl.thw, wl.cu_seqlens, wl.scale)
    return dev, (out, dq, dk, dv)


@pytest.mark.parametrize("name", list(CASES))
def test_temporal_attention_matches_oracle(name):
    wl = CASES[name]
    dev, gpu = _run(_binding(), wl)
    _check(wl, gpu, dev)


def test_single_frame_clip_copies_values_and_has_zero_qk_gradients():
    wl = CASES["t128"]
    dev, (out, dq, dk, dv) = _run(_binding(), wl)
    a, b = int(wl.cu_seqlens[1]), int(wl.cu_seqlens[2])      # the (1,2,3) clip
    assert np.array_equal(U.to_bits(out[a:b]), U.to_bits(dev["v"][a:b]))
    assert not np.any(U.to_f64(dq[a:b])) and not np.any(U.to_f64(dk[a:b]))
    assert np.array_equal(U.to_bits(dv[a:b]), U.to_bits(dev["dout"][a:b]))


LONG = {
    # more than 32 frames (Section 4.6: videos of hundreds of frames): 33, 48, 121 frames, block
    # multiples (64, 96) and short clips, an empty and a single-frame one in the same call
    "t128_33_48": W.Workload("t128_33_48", ((33, 2, 3), (48, 1, 5), (4, 3, 3), (0, 1, 1), (1, 2, 2), (64, 1, 2)), 3, 128,
                             (32, 48, 48), seed=35),
    "t128_121": W.Workload("t128_121", ((121, 3, 2), (96, 1, 1), (17, 2, 2)), 2, 128, (32, 48, 48), seed=36),
    "t64_long": W.Workload("t64_100", ((100, 2, 2), (33, 1, 3), (65, 1, 1), (2, 2, 2)), 2, 64, (16, 24, 24), seed=37),
    "t128_300": W.Workload("t128_300", ((300, 1, 2),), 1, 128, (32, 48, 48), seed=38),
}


@pytest.mark.parametrize("name", list(LONG))
def test_more_than_thirty_two_frames(name):
    wl = LONG[name]
    dev, gpu = _run(_binding(), wl)
    _check(wl, gpu, dev)


def test_long_clip_statistics_do_not_leak_into_dq():
    # with more than 32 frames the dq rows carry the queries' statistics while the call runs; afterwards
    # every dq element is a gradient, also after a second call into the same buffers
    import torch
    wl = LONG["t128_33_48"]
    b = _binding()
    inp = W.make_inputs(wl)
    dev = {n: U.to_device(inp[n]) for n in ("q", "k", "v", "dout")}
    dq, dk, dv = (torch.full_like(dev["q"], float("nan")) for _ in range(3))
    for _ in range(2):
        b.vfm_tattn_bwd(dev["q"], dev["k"], dev["v"], dev["dout"], wl.thw, wl.cu_seqlens, wl.scale, dq=dq, dk=dk, dv=dv)
    host = {n: U.to_f64(t) for n, t in dev.items()}
    g_ref = orc.temporal_attn_bwd(host["q"], host["k"], host["v"], host["dout"], wl.thw, wl.cu_seqlens, wl.scale)
    for nm, g, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), g_ref):
        assert U.rel_rms(U.to_f64(g), ref) <= U.TOL_GRAD_RELRMS, nm
        U.assert_rows_close(nm, U.to_f64(g), ref, U.TOL_GRAD_RELRMS)


def test_single_frame_clip_in_a_long_call():
    # the 32-row kernels serve every clip of a call that has a long one
    wl = CASES["t128_long"]
    dev, (out, dq, dk, dv) = _run(_binding(), wl)
    a, b = int(wl.cu_seqlens[5]), int(wl.cu_seqlens[6])      # the (1,3,1) clip
    assert np.array_equal(U.to_bits(out[a:b]), U.to_bits(dev["v"][a:b]))
    assert not np.any(U.to_f64(dq[a:b])) and not np.any(U.to_f64(dk[a:b]))
    assert np.array_equal(U.to_bits(dv[a:b]), U.to_bits(dev["dout"][a:b]))


def test_full_size_c4_every_element():
    """The 56,320-token latent (16 frames x 3,520 pixels), 32 heads: every element of out, dq,
    dk, dv against the oracle, four heads at a time."""
    wl = W.WORKLOADS["C4"]
    dev, gpu = _run(_binding(), wl)
    for h0 in range(0, wl.n_heads, 4):
        _check(wl, gpu, dev, heads=range(h0, h0 + 4))
