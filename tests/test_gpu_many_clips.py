"""Calls with more clips than one kernel-argument table holds (256; 128 cross-attention
sequences): the library cuts them into consecutive launches over runs of clips.  Section 3.1
packs images and videos together and Table 1 trains at a 73,728-token context: 256-token images
alone are 288 clips; the spatial view of Section 4.6 makes every latent frame a sequence."""
import numpy as np
import pytest

from oracle import vfm_oracle as orc
from paper_2503_12964_amd import workloads as W
from tests import parity_utils as U
from tests.test_gpu_parity import _assert_parity, _binding, _run_fwd_bwd

pytestmark = pytest.mark.gpu


def test_288_images_of_256_tokens():
    # a 73,728-token context filled with 16 x 16 images: two runs (256 + 32 clips)
    wl = W.Workload("images288", tuple((1, 16, 16) for _ in range(288)), 2, 128, (32, 48, 48), seed=78)
    assert wl.total_tokens == 73728
    gpu, host = _run_fwd_bwd(wl, rope=True)
    _assert_parity(wl, gpu, host)


def test_short_sequences_one_launch_equals_two_passes():
    # Packs whose sequences all have at most 1,024 rows run dK/dV and dQ units from one grid; one
    # longer clip in the pack sends it through the two separate kernels.  Both run the same unit
    # code on the same rows, so the short clips' gradients must agree bit for bit.
    import torch
    short = tuple((1, 16, 16) for _ in range(5)) + ((1, 3, 7), (2, 9, 17), (1, 32, 32), (1, 1, 1), (1, 20, 45))
    wl_a = W.Workload("short", short, 3, 128, (32, 48, 48), seed=85)
    wl_b = W.Workload("short+long", short + ((1, 33, 32),), 3, 128, (32, 48, 48), seed=85)
    assert max(wl_a.seqlens) <= 1024 < max(wl_b.seqlens)
    b = _binding()
    inp = W.make_inputs(wl_b)
    n = wl_a.total_tokens
    dev_b = {k: U.to_device(x) for k, x in inp.items()}
    dev_a = {k: t[:n].contiguous() for k, t in dev_b.items()}
    res = []
    for wl, dev in ((wl_a, dev_a), (wl_b, dev_b)):
        out, lse = b.vfm_attn_fwd(dev["q"], dev["k"], dev["v"], wl.cu_seqlens, wl.scale)
        res.append(b.vfm_attn_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], wl.cu_seqlens, wl.scale))
    for nm, ga, gb in zip(("dq", "dk", "dv"), *res):
        assert torch.equal(ga.view(torch.int16), gb[:n].view(torch.int16)), nm
    host = tuple(U.to_f64(dev_a[k]) for k in ("q", "k", "v", "dout"))
    g_ref = orc.attn_bwd(*host, wl_a.cu_seqlens, wl_a.scale)
    for nm, g, ref in zip(("dq", "dk", "dv"), res[0], g_ref):
        assert U.rel_rms(U.to_f64(g), ref) <= U.TOL_GRAD_RELRMS, nm


def test_600_mixed_clips():
    # three runs; empty, one-token and tile-boundary clips fall on both sides of the cuts
    rng = np.random.default_rng(17)
    grids = []
    for i in range(600):
        kind = rng.integers(0, 8)
        if kind == 0:
            grids.append((0, 1, 1))
        elif kind == 1:
            grids.append((1, 1, 1))
        elif kind == 2:
            grids.append((1, 1, int(rng.choice([31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257]))))
        else:
            grids.append((int(rng.integers(1, 4)), int(rng.integers(1, 7)), int(rng.integers(1, 9))))
    grids[255], grids[256], grids[511], grids[512] = (2, 9, 17), (1, 1, 300), (0, 1, 1), (3, 8, 8)
    for hd, dims in ((128, (32, 48, 48)), (64, (16, 24, 24))):
        wl = W.Workload(f"mixed600_{hd}", tuple(grids), 3, hd, dims, seed=79)
        gpu, host = _run_fwd_bwd(wl, rope=True)
        _assert_parity(wl, gpu, host, relative_maxabs=True)


def test_spatial_view_of_many_frames():
    # 5 clips of 64 to 100 latent frames with few tokens each: 402 per-frame sequences
    wl = W.Workload("frames402", ((64, 4, 6), (100, 3, 5), (70, 5, 5), (88, 2, 9), (80, 6, 3)), 2, 128, (32, 48, 48),
                    seed=80)
    b = _binding()
    inp = W.make_inputs(wl)
    q, k, v, do = (U.to_device(inp[n]) for n in ("q", "k", "v", "dout"))
    b.vfm_rope3d(q, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    b.vfm_rope3d(k, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    cu = wl.spatial_cu_seqlens
    assert len(cu) - 1 == 402
    out, lse = b.vfm_attn_fwd(q, k, v, cu, wl.scale)
    dq, dk, dv = b.vfm_attn_bwd(q, k, v, out, lse, do, cu, wl.scale)
    frames = W.Workload("frames", tuple((1, 1, int(n)) for n in np.diff(cu)), wl.n_heads, wl.head_dim,
                        wl.rope_dims, wl.seed)
    _assert_parity(frames, (out, lse, dq, dk, dv), tuple(U.to_f64(t) for t in (q, k, v, do)), relative_maxabs=True)


def test_rope_and_qknorm_over_many_clips():
    import torch
    rng = np.random.default_rng(18)
    grids = tuple((int(rng.integers(0, 4)), int(rng.integers(1, 6)), int(rng.integers(1, 6))) for _ in range(700))
    wl = W.Workload("rope700", grids, 3, 128, (32, 48, 48), seed=81)
    b = _binding()
    inp = W.make_inputs(wl, tensors=("q", "dout"))
    for inverse in (False, True):
        x = U.to_device(inp["q"])
        b.vfm_rope3d(x, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta, inverse=inverse)
        xin = U.bits_to_f64(inp["q"])
        want = orc.rope3d(xin, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta, inverse=inverse)
        tol = 2.0 ** -8 * np.abs(want) + 1e-6 * np.abs(xin).max()
        assert np.all(np.abs(U.to_f64(x) - want) <= tol)
    gain = W.norm_gain(wl)
    gain_d = torch.from_numpy(gain).cuda()
    x, dy = U.to_device(inp["q"]), U.to_device(inp["dout"])
    y = b.vfm_qknorm_rope3d(x, gain_d, 1e-6, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta,
                            y=U.to_device(np.zeros_like(inp["q"])))
    want = orc.qknorm_rope3d(U.bits_to_f64(inp["q"]), gain, 1e-6, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    assert np.all(np.abs(U.to_f64(y) - want) <= 2.0 ** -8 * np.abs(want) + 4e-6 * np.abs(want).max())
    dx, dgain = b.vfm_qknorm_rope3d_bwd(x, gain_d, 1e-6, dy, wl.thw, wl.cu_seqlens, wl.rope_dims, wl.theta)
    dx_ref, dg_ref = orc.qknorm_rope3d_bwd(U.bits_to_f64(inp["q"]), gain, 1e-6, U.bits_to_f64(inp["dout"]), wl.thw,
                                           wl.cu_seqlens, wl.rope_dims, wl.theta)
    assert np.all(np.abs(U.to_f64(dx) - dx_ref) <= 2.0 ** -8 * np.abs(dx_ref) + 4e-6 * np.abs(dx_ref).max())
    assert np.max(np.abs(U.to_f64(dgain) - dg_ref)) <= 2e-4 * np.abs(dg_ref).max()     # summed over all three runs


def test_cross_attention_over_many_sequences():
    # 300 sequences (three runs of 128, 128, 44); long query ranges against a few keys take the
    # query-split dK/dV pass, whose accumulators must stay inside their own run's key rows
    rng = np.random.default_rng(19)
    nq = rng.integers(0, 40, size=300)
    nk = np.where(nq > 0, rng.integers(1, 90, size=300), rng.integers(0, 3, size=300))
    nq[5], nk[5] = 3000, 40
    nq[130], nk[130] = 2500, 7
    nq[290], nk[290] = 2800, 130
    cu_q = np.concatenate([[0], np.cumsum(nq)]).astype(np.int32)
    cu_kv = np.concatenate([[0], np.cumsum(nk)]).astype(np.int32)
    b = _binding()
    heads, hd = 1, 128        # one head: fewer than 256 key-tile workgroups per run, so the split pass is taken
    tq, tk = int(cu_q[-1]), int(cu_kv[-1])
    bits = {n: W.f32_to_bf16_bits(W.normal_f32(83, n, (t, heads, hd)))
            for n, t in (("q", tq), ("k", tk), ("v", tk), ("dout", tq))}
    dev = {n: U.to_device(x) for n, x in bits.items()}
    scale = 1.0 / np.sqrt(hd)
    out, lse = b.vfm_xattn_fwd(dev["q"], dev["k"], dev["v"], cu_q, cu_kv, scale)
    dq, dk, dv = b.vfm_xattn_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], cu_q, cu_kv, scale)
    host = {n: U.to_f64(t) for n, t in dev.items()}
    o_ref, l_ref = orc.xattn_fwd(host["q"], host["k"], host["v"], cu_q, cu_kv, scale)
    g_ref = orc.xattn_bwd(host["q"], host["k"], host["v"], host["dout"], cu_q, cu_kv, scale)
    o = U.to_f64(out)
    assert np.max(np.abs(o - o_ref) / np.maximum(1.0, np.abs(o_ref))) <= U.TOL_OUT_MAXABS
    assert U.rel_rms(o, o_ref) <= U.TOL_OUT_RELRMS
    U.assert_rows_close("out", o, o_ref, U.TOL_OUT_RELRMS)
    assert U.max_abs(U.to_f64(lse), l_ref) <= U.TOL_LSE_MAXABS
    for nm, g, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), g_ref):
        got = U.to_f64(g)
        assert U.rel_rms(got, ref) <= U.TOL_GRAD_RELRMS, nm
        U.assert_rows_close(nm, got, ref, U.TOL_GRAD_RELRMS)


def test_temporal_attention_over_many_clips():
    rng = np.random.default_rng(20)
    grids = tuple((int(rng.integers(0, 9)), int(rng.integers(1, 4)), int(rng.integers(1, 4))) for _ in range(300))
    grids = grids[:255] + ((20, 2, 2), (32, 1, 3)) + grids[257:]        # long clips on both sides of the cut
    wl = W.Workload("t300", grids, 2, 128, (32, 48, 48), seed=84)
    b = _binding()
    inp = W.make_inputs(wl)
    dev = {n: U.to_device(inp[n]) for n in ("q", "k", "v", "dout")}
    out = b.vfm_tattn_fwd(dev["q"], dev["k"], dev["v"], wl.thw, wl.cu_seqlens, wl.scale)
    dq, dk, dv = b.vfm_tattn_bwd(dev["q"], dev["k"], dev["v"], dev["dout"], wl.thw, wl.cu_seqlens, wl.scale)
    host = {n: U.to_f64(t) for n, t in dev.items()}
    o_ref = orc.temporal_attn_fwd(host["q"], host["k"], host["v"], wl.thw, wl.cu_seqlens, wl.scale)
    g_ref = orc.temporal_attn_bwd(host["q"], host["k"], host["v"], host["dout"], wl.thw, wl.cu_seqlens, wl.scale)
    assert U.rel_rms(U.to_f64(out), o_ref) <= U.TOL_OUT_RELRMS
    U.assert_rows_close("out", U.to_f64(out), o_ref, U.TOL_OUT_RELRMS)
    for nm, g, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), g_ref):
        assert U.rel_rms(U.to_f64(g), ref) <= U.TOL_GRAD_RELRMS, nm
        U.assert_rows_close(nm, U.to_f64(g), ref, U.TOL_GRAD_RELRMS)
