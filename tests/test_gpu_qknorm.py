"""GPU parity of the fused per-head normalisation + 3D RoPE (forward and backward) against the
fp64 oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import vfm_oracle as orc
from paper_2503_12964_amd import workloads as W
from tests import parity_utils as U
from tests.test_gpu_parity import SMALL, _binding

pytestmark = pytest.mark.gpu

EPS = 1e-6
# y and dx are one bf16 rounding of an fp32 result: relative RMS of a rounding is 2^-9/sqrt(3) = 1.1e-3
TOL_RELRMS = 2.5e-3
# dgain: fp32 sums of products of values that are exact on both sides; only summation order differs
TOL_DGAIN_REL = 2e-4


def _inputs(wl, scale=1.0):
    import torch
    inp = W.make_inputs(wl, tensors=("q", "dout"))
    xb = inp["q"]
    if scale != 1.0:    # un-normalised activations: the kernel must not care about the magnitude
        xb = W.f32_to_bf16_bits(W.bf16_bits_to_f32(xb) * np.float32(scale))
    gain = W.norm_gain(wl)
    return xb, inp["dout"], gain, torch.from_numpy(gain).cuda()


def _elementwise_ok(got, want, scale_ref):
    # one bf16 ulp of the exact value plus fp32 rounding of the sums and products
    tol = 2.0 ** -8 * np.abs(want) + 4e-6 * scale_ref
    assert np.all(np.abs(got - want) <= tol), f"max excess {np.max(np.abs(got - want) - tol)}"


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("scale", [1.0, 37.5])
def test_forward_matches_oracle(name, scale):
    wl = SMALL[name]
    b = _binding()
    xb, _, gain, gain_d = _inputs(wl, scale)
    x = U.to_device(xb)
    y = b.vfm_qknorm_rope3d(x, gain_d, EPS, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta,
                            y=U.to_device(np.zeros_like(xb)))
    want = orc.qknorm_rope3d(U.bits_to_f64(xb), gain, EPS, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    got = U.to_f64(y)
    _elementwise_ok(got, want, np.abs(want).max())
    assert U.rel_rms(got, want) <= TOL_RELRMS
    assert np.array_equal(U.to_bits(x), xb)          # out of place: x untouched
    # in place gives the same bits
    b.vfm_qknorm_rope3d(x, gain_d, EPS, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    assert np.array_equal(U.to_bits(x), U.to_bits(y))


@pytest.mark.parametrize("name", list(SMALL))
def test_backward_matches_oracle(name):
    wl = SMALL[name]
    b = _binding()
    xb, dyb, gain, gain_d = _inputs(wl, 3.0)
    x, dy = U.to_device(xb), U.to_device(dyb)
    dx, dgain = b.vfm_qknorm_rope3d_bwd(x, gain_d, EPS, dy, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    dx_ref, dg_ref = orc.qknorm_rope3d_bwd(U.bits_to_f64(xb), gain, EPS, U.bits_to_f64(dyb), wl.thw,
                                           wl.cu_seqlens, wl.rope_dims, wl.theta)
    got = U.to_f64(dx)
    _elementwise_ok(got, dx_ref, np.abs(dx_ref).max())
    assert U.rel_rms(got, dx_ref) <= TOL_RELRMS
    dg = U.to_f64(dgain)
    assert np.max(np.abs(dg - dg_ref)) <= TOL_DGAIN_REL * np.abs(dg_ref).max()
    # dx may overwrite dy
    dx2, dgain2 = b.vfm_qknorm_rope3d_bwd(x, gain_d, EPS, dy, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta, dx=dy)
    assert np.array_equal(U.to_bits(dx2), U.to_bits(dx))
    assert np.max(np.abs(U.to_f64(dgain2) - dg)) <= 1e-5 * np.abs(dg).max()
    # dx must not be x
    with pytest.raises(b.VfmError):
        b.vfm_qknorm_rope3d_bwd(x, gain_d, EPS, dy, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta, dx=x)


def test_unit_gain_unit_rms_input_equals_plain_rope_kernel():
    # a row whose mean square is exactly 1 (entries +-1) is left alone by the normalisation:
    # the fused kernel must then agree with vfm_rope3d bit for bit
    import torch
    wl = SMALL["ragged128"]
    b = _binding()
    sign = np.where(W.bf16_bits_to_f32(W.make_inputs(wl, tensors=("q",))["q"]) >= 0, 1.0, -1.0).astype(np.float32)
    xb = W.f32_to_bf16_bits(sign)
    ones = torch.ones(wl.head_dim, dtype=torch.float32, device="cuda")
    y = b.vfm_qknorm_rope3d(U.to_device(xb), ones, 0.0, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    r = b.vfm_rope3d(U.to_device(xb), wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    assert np.array_equal(U.to_bits(y), U.to_bits(r))


def test_full_size_c4_every_element():
    """C4 shape (56,320 tokens, 32 heads, head_dim 128), the launch configuration bench.py times.
    Heads are independent except in dgain, so the oracle runs on four heads at a time and
    covers every element of y and dx and the complete dgain sum."""
    wl = W.WORKLOADS["C4"]
    b = _binding()
    xb, dyb, gain, gain_d = _inputs(wl)
    x, dy = U.to_device(xb), U.to_device(dyb)
    y = b.vfm_qknorm_rope3d(x, gain_d, EPS, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta,
                            y=U.to_device(np.zeros_like(xb)))
    dx, dgain = b.vfm_qknorm_rope3d_bwd(x, gain_d, EPS, dy, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    y_bits, dx_bits = U.to_bits(y), U.to_bits(dx)
    dg_ref = np.zeros(wl.head_dim)
    err2 = {"y": 0.0, "dx": 0.0}
    ref2 = {"y": 0.0, "dx": 0.0}
    for h0 in range(0, wl.n_heads, 4):
        hs = slice(h0, h0 + 4)
        x64, dy64 = U.bits_to_f64(xb[:, hs]), U.bits_to_f64(dyb[:, hs])
        y_ref = orc.qknorm_rope3d(x64, gain, EPS, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
        dx_ref, dg = orc.qknorm_rope3d_bwd(x64, gain, EPS, dy64, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
        dg_ref += dg
        for key, got_bits, want in (("y", y_bits[:, hs], y_ref), ("dx", dx_bits[:, hs], dx_ref)):
            got = U.bits_to_f64(got_bits)
            _elementwise_ok(got, want, np.abs(want).max())
            err2[key] += float(np.sum((got - want) ** 2))
            ref2[key] += float(np.sum(want ** 2))
    for key in err2:
        assert np.sqrt(err2[key] / ref2[key]) <= TOL_RELRMS
    dg = U.to_f64(dgain)
    assert np.max(np.abs(dg - dg_ref)) <= TOL_DGAIN_REL * np.abs(dg_ref).max()
