"""GPU parity of packed cross-attention (separate query and key/value boundaries) against the
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


def _draw(seed, name, shape):
    return W.f32_to_bf16_bits(W.normal_f32(seed, name, shape))


def _run(b, cu_q, cu_kv, heads, hd, seed):
    tq, tk = int(cu_q[-1]), int(cu_kv[-1])
    bits = {"q": _draw(seed, "q", (tq, heads, hd)), "k": _draw(seed, "k", (tk, heads, hd)),
            "v": _draw(seed, "v", (tk, heads, hd)), "dout": _draw(seed, "dout", (tq, heads, hd))}
    dev = {n: U.to_device(x) for n, x in bits.items()}
    scale = 1.0 / np.sqrt(hd)
    out, lse = b.vfm_xattn_fwd(dev["q"], dev["k"], dev["v"], cu_q, cu_kv, scale)
    dq, dk, dv = b.vfm_xattn_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], cu_q, cu_kv, scale)
    return dev, (out, lse, dq, dk, dv), scale


def _assert(gpu, dev, cu_q, cu_kv, scale, heads=None):
    out, lse, dq, dk, dv = gpu
    hs = slice(None) if heads is None else list(heads)
    host = {n: U.to_f64(t[:, hs, :]) for n, t in dev.items()}
    o_ref, l_ref = orc.xattn_fwd(host["q"], host["k"], host["v"], cu_q, cu_kv, scale)
    g_ref = orc.xattn_bwd(host["q"], host["k"], host["v"], host["dout"], cu_q, cu_kv, scale)
    o = U.to_f64(out[:, hs, :])
    assert np.all(np.isfinite(o))
    # few keys make outputs O(|v|): bound the error relative to max(1, |ref|) as for peaky softmax
    assert np.max(np.abs(o - o_ref) / np.maximum(1.0, np.abs(o_ref))) <= U.TOL_OUT_MAXABS
    assert U.rel_rms(o, o_ref) <= U.TOL_OUT_RELRMS
    U.assert_rows_close("out", o, o_ref, U.TOL_OUT_RELRMS)
    # queries of empty sequences do not exist, so every lse entry is defined
    assert U.max_abs(U.to_f64(lse[hs, :]), l_ref) <= U.TOL_LSE_MAXABS
    for nm, g, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), g_ref):
        got = U.to_f64(g[:, hs, :])
        r = U.rel_rms(got, ref)
        assert r <= U.TOL_GRAD_RELRMS, (nm, r)
        U.assert_rows_close(nm, got, ref, U.TOL_GRAD_RELRMS)       # every (token, head) row
    return g_ref


RAGGED = {
    # a sequence with keys and no queries, one with a single query, one with a single key,
    # key counts around the 32-row unit and the 64/128-row tiles, query counts around 256
    "x128": (np.array([0, 300, 300, 301, 650, 891, 1403]), np.array([0, 77, 90, 123, 124, 253, 510]), 3, 128),
    "x64": (np.array([0, 257, 263, 600]), np.array([0, 33, 161, 225]), 2, 64),
}


@pytest.mark.parametrize("name", list(RAGGED))
def test_ragged_cross_attention_matches_oracle(name):
    cu_q, cu_kv, heads, hd = RAGGED[name]
    b = _binding()
    dev, gpu, scale = _run(b, cu_q, cu_kv, heads, hd, seed=21)
    g_ref = _assert(gpu, dev, cu_q, cu_kv, scale)
    if name == "x128":      # keys 77..89 belong to the sequence without queries
        assert not np.any(U.to_f64(gpu[3][77:90])) and not np.any(U.to_f64(gpu[4][77:90]))
        assert not np.any(g_ref[1][77:90])


def test_equal_ranges_are_bitwise_the_self_attention_result():
    b = _binding()
    cu = np.array([0, 300, 301, 301, 891])
    dev, gpu, scale = _run(b, cu, cu, 3, 128, seed=22)
    out, lse = b.vfm_attn_fwd(dev["q"], dev["k"], dev["v"], cu, scale)
    dq, dk, dv = b.vfm_attn_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], cu, scale)
    import torch
    for a, c in zip(gpu, (out, lse, dq, dk, dv)):
        assert torch.equal(a, c)


def test_queries_without_keys_are_an_error():
    b = _binding()
    import torch
    q = torch.zeros((8, 1, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(b.VfmError):
        b.vfm_xattn_fwd(q, q, q, [0, 4, 8], [0, 8, 8], 0.125)


@pytest.mark.parametrize("cu_q,cu_kv,heads,check", [
    # the 56,320-token latent attending to a 512-token text embedding, 32 heads, every head checked
    (np.array([0, 56320]), np.array([0, 512]), 32, None),
    # classifier-free-guidance style pair: two 4,096-token latents, prompts of 226 and 77 tokens
    (np.array([0, 4096, 8192]), np.array([0, 226, 303]), 16, None),
])
def test_paper_shaped_cross_attention(cu_q, cu_kv, heads, check):
    b = _binding()
    dev, gpu, scale = _run(b, cu_q, cu_kv, heads, 128, seed=23)
    for h0 in range(0, heads, 8):       # oracle on eight heads at a time (memory)
        _assert(gpu, dev, cu_q, cu_kv, scale, heads=range(h0, min(h0 + 8, heads)))
