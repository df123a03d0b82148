"""GPU parity: libvfm (through the C ABI) against the fp64 oracle, element by element."""
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


def _custom(name, grids, heads, hd, dims, seed):
    return W.Workload(name, tuple(grids), heads, hd, dims, seed=seed)


SMALL = {
    "C1": W.WORKLOADS["C1"],
    # ragged clips at head_dim 128: several 256-row tiles, tails, a 1-token clip and an empty one
    "ragged128": _custom("ragged128", [(3, 10, 10), (1, 1, 1), (1, 7, 11), (0, 1, 1), (3, 9, 19)], 3, 128,
                         (32, 48, 48), 11),
    # ragged clips at head_dim 64
    "ragged64": _custom("ragged64", [(2, 9, 15), (1, 5, 13), (1, 1, 2)], 2, 64, (16, 24, 24), 12),
    # clip lengths around the kernels' 32-key blocks and 64-key tiles: 32, 64, 96, 128, 33, 65, 31, 63
    "block_edges": _custom("block_edges", [(1, 4, 8), (1, 8, 8), (1, 8, 12), (2, 8, 8), (1, 3, 11), (1, 5, 13),
                                           (1, 1, 31), (1, 7, 9)], 2, 128, (32, 48, 48), 13),
}


def _check_rope(wl, inverse=False):
    b = _binding()
    bits = W.make_inputs(wl, tensors=("q",))["q"]
    x = U.to_device(bits)
    b.vfm_rope3d(x, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta, inverse=inverse)
    got = U.to_f64(x)
    xin = U.bits_to_f64(bits)
    want = orc.rope3d(xin, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta, inverse=inverse)
    # one bf16 ulp of the exact value, plus fp32 rounding of the products before the subtraction
    tol = 2.0 ** -8 * np.abs(want) + 1e-6 * np.abs(xin).max()
    assert np.all(np.abs(got - want) <= tol), f"max excess {np.max(np.abs(got - want) - tol)}"
    assert U.rel_rms(got, want) <= U.TOL_ROPE_RELRMS
    return x, bits


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("inverse", [False, True])
def test_rope_matches_oracle(name, inverse):
    _check_rope(SMALL[name], inverse)


def test_rope_identity_at_origin_and_norms():
    wl = SMALL["ragged128"]
    x, bits = _check_rope(wl)
    got = U.to_bits(x)
    for a, n in zip(wl.cu_seqlens[:-1], wl.seqlens):
        if n:
            assert np.array_equal(got[a], bits[a])           # position (0,0,0): untouched bit patterns


def _run_fwd_bwd(wl, gain=1.0, rope=False):
    b = _binding()
    inp = W.make_inputs(wl, gain_qk=gain)
    q, k, v, do = (U.to_device(inp[n]) for n in ("q", "k", "v", "dout"))
    if rope:
        b.vfm_rope3d(q, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
        b.vfm_rope3d(k, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    out, lse = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    dq, dk, dv = b.vfm_attn_bwd(q, k, v, out, lse, do, wl.cu_seqlens, wl.scale)
    # the oracle sees exactly the bf16 values the attention kernels saw
    q64, k64, v64, do64 = (U.to_f64(t) for t in (q, k, v, do))
    return (out, lse, dq, dk, dv), (q64, k64, v64, do64)


def _assert_parity(wl, gpu, host, relative_maxabs=False):
    out, lse, dq, dk, dv = gpu
    q64, k64, v64, do64 = host
    o_ref, l_ref = orc.attn_fwd(q64, k64, v64, wl.cu_seqlens, wl.scale)
    g_ref = orc.attn_bwd(q64, k64, v64, do64, wl.cu_seqlens, wl.scale)
    o = U.to_f64(out)
    assert np.all(np.isfinite(o))
    if relative_maxabs:
        # peaky softmax: outputs are O(|v|) instead of O(N^-1/2), so one bf16 rounding of the
        # output alone exceeds an absolute 1e-2; bound the error relative to max(1, |ref|)
        assert np.max(np.abs(o - o_ref) / np.maximum(1.0, np.abs(o_ref))) <= U.TOL_OUT_MAXABS
    else:
        assert U.max_abs(o, o_ref) <= U.TOL_OUT_MAXABS
    assert U.rel_rms(o, o_ref) <= U.TOL_OUT_RELRMS
    U.assert_rows_close("out", o, o_ref, U.TOL_OUT_RELRMS)
    assert U.max_abs(U.to_f64(lse), l_ref) <= U.TOL_LSE_MAXABS
    # The backward forms Delta = rowsum(dO o out) from the bf16 `out` it is handed (clips of at most
    # 32 keys aside).  Where dS cancels almost completely (peaky softmax) that rounding shows in single
    # rows of dq, dk although the tensor bound holds, so a row may sit within the per-row bound of
    # the exact gradient or of the gradient that the same Delta from the same `out` gives; a
    # damaged row is far from both.
    g_met = orc.attn_bwd(q64, k64, v64, do64, wl.cu_seqlens, wl.scale, out=o)
    for name, g, ref, met in zip(("dq", "dk", "dv"), (dq, dk, dv), g_ref, g_met):
        g64 = U.to_f64(g)
        assert np.all(np.isfinite(g64)), name
        assert U.rel_rms(g64, ref) <= U.TOL_GRAD_RELRMS, (name, U.rel_rms(g64, ref))
        U.assert_rows_close(name, g64, ref, U.TOL_GRAD_RELRMS, also=met)     # every (token, head) row


@pytest.mark.parametrize("name", list(SMALL))
def test_attention_fwd_bwd_matches_oracle(name):
    wl = SMALL[name]
    gpu, host = _run_fwd_bwd(wl)
    _assert_parity(wl, gpu, host)


@pytest.mark.parametrize("name", ["C1", "ragged128"])
def test_attention_with_rope_end_to_end(name):
    # per call: attention is checked against the oracle fed the GPU's own bf16 RoPE output
    wl = SMALL[name]
    gpu, host = _run_fwd_bwd(wl, rope=True)
    _assert_parity(wl, gpu, host)


def test_spatial_attention_view():
    # Section 4.6: spatial attention re-reads the packed clips as one sequence per latent frame;
    # RoPE still uses the clips' own grids, attention uses the per-frame boundaries
    wl = SMALL["ragged128"]
    b = _binding()
    inp = W.make_inputs(wl)
    q, k, v, do = (U.to_device(inp[n]) for n in ("q", "k", "v", "dout"))
    b.vfm_rope3d(q, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    b.vfm_rope3d(k, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    cu = wl.spatial_cu_seqlens
    assert cu.tolist() == [0, 100, 200, 300, 301, 378, 549, 720, 891]
    out, lse = b.vfm_attn_fwd(q, k, v, cu, wl.scale)
    dq, dk, dv = b.vfm_attn_bwd(q, k, v, out, lse, do, cu, wl.scale)
    frames = W.Workload("frames", tuple((1, 1, int(n)) for n in np.diff(cu)), wl.n_heads, wl.head_dim,
                        wl.rope_dims, wl.seed)
    _assert_parity(frames, (out, lse, dq, dk, dv), tuple(U.to_f64(t) for t in (q, k, v, do)))


def test_peaky_softmax_running_max():
    # q, k scaled by 4: scores ~ N(0, 16^2); exercises the running-max update path
    wl = SMALL["ragged128"]
    gpu, host = _run_fwd_bwd(wl, gain=4.0)
    _assert_parity(wl, gpu, host, relative_maxabs=True)


@pytest.mark.parametrize("ramp_to", [8.0, 40.0])
def test_softmax_reference_moves_with_growing_scores(ramp_to):
    # key magnitude grows along each clip, so later key units keep exceeding the forward
    # kernel's softmax reference point: with ramp_to = 8 it has to move several times, with
    # 40 the exponentials taken against the stale reference overflow to inf before it moves
    import torch
    wl = SMALL["ragged128"]
    b = _binding()
    inp = W.make_inputs(wl)
    q, k, v, do = (U.to_device(inp[n]) for n in ("q", "k", "v", "dout"))
    ramp = torch.linspace(1.0, ramp_to, wl.total_tokens, device=k.device)
    k = (k.float() * ramp[:, None, None]).to(torch.bfloat16)
    out, lse = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    dq, dk, dv = b.vfm_attn_bwd(q, k, v, out, lse, do, wl.cu_seqlens, wl.scale)
    host = tuple(U.to_f64(t) for t in (q, k, v, do))
    _assert_parity(wl, (out, lse, dq, dk, dv), host, relative_maxabs=True)


def test_forward_is_bitwise_reproducible():
    wl = SMALL["ragged128"]
    b = _binding()
    inp = W.make_inputs(wl)
    q, k, v = (U.to_device(inp[n]) for n in ("q", "k", "v"))
    o1, l1 = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    o2, l2 = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    assert np.array_equal(U.to_bits(o1), U.to_bits(o2))
    assert np.array_equal(l1.cpu().numpy(), l2.cpu().numpy())


def test_backward_is_bitwise_reproducible():
    # no atomics anywhere in the self-attention backward: two calls give identical bits
    wl = SMALL["ragged128"]
    b = _binding()
    inp = W.make_inputs(wl)
    q, k, v, do = (U.to_device(inp[n]) for n in ("q", "k", "v", "dout"))
    out, lse = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    g1 = b.vfm_attn_bwd(q, k, v, out, lse, do, wl.cu_seqlens, wl.scale)
    g2 = b.vfm_attn_bwd(q, k, v, out, lse, do, wl.cu_seqlens, wl.scale)
    for a, c in zip(g1, g2):
        assert np.array_equal(U.to_bits(a), U.to_bits(c))


@pytest.mark.parametrize("seed", [5469, 1, 2, 3])
def test_two_token_clip_meets_the_gradient_bound(seed):
    # In a clip of two tokens dQ and dK are small by cancellation (dS_i1 = -dS_i2).  With Delta
    # taken from the bf16 `out` this very call (seed 5469, found by a random sweep) was off by 2%
    # in dq and dk; for clips of at most 32 keys the backward now forms Delta as sum_j P_ij dP_ij,
    # and the stated bound holds, for the tensor and for every row.
    wl = W.Workload("two_tokens", ((1, 1, 2), (0, 1, 1)), 1, 128, (32, 48, 48), seed=seed)
    gpu, host = _run_fwd_bwd(wl, rope=True)
    _assert_parity(wl, gpu, host, relative_maxabs=True)


def test_tiny_clips_of_every_length_up_to_forty():
    # clip lengths 1..40 in one call, both sides of the 32-key limit of the exact-Delta path
    wl = _custom("tiny_clips", [(1, 1, n) for n in range(1, 41)], 2, 128, (32, 48, 48), 31)
    gpu, host = _run_fwd_bwd(wl, rope=True)
    _assert_parity(wl, gpu, host, relative_maxabs=True)
    wl = _custom("tiny_clips64", [(1, 1, n) for n in (1, 2, 3, 5, 8, 13, 21, 32, 33, 34)], 3, 64, (16, 24, 24), 32)
    gpu, host = _run_fwd_bwd(wl, rope=True)
    _assert_parity(wl, gpu, host, relative_maxabs=True)


def test_closed_forms_on_gpu():
    import torch
    b = _binding()
    # single-token clips return V; zero queries return the clip mean of V
    wl = _custom("ones", [(1, 1, 1)] * 5 + [(1, 4, 10)], 2, 128, (32, 48, 48), 13)
    inp = W.make_inputs(wl)
    q, k, v = (U.to_device(inp[n]) for n in ("q", "k", "v"))
    out, lse = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    assert np.array_equal(U.to_bits(out)[:5], inp["v"][:5])
    q.zero_()
    out, lse = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    mean_v = U.bits_to_f64(inp["v"])[5:].mean(0)
    assert U.max_abs(U.to_f64(out)[5:], np.broadcast_to(mean_v, (40,) + mean_v.shape)) <= 2.0 ** -8
    assert U.max_abs(U.to_f64(lse)[:, 5:], np.log(40.0)) <= 1e-5
    torch.cuda.synchronize()
