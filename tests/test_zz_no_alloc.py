"""The entry point that allocates nothing: vfm_attn_bwd_noalloc keeps the backward's statistics
in an array built into the library's device code instead of a caller workspace.  It runs the
same kernels as vfm_attn_bwd, so its gradients must be bitwise those of vfm_attn_bwd (which the
other parity tests hold against the fp64 oracle), on two calls in a row, the second with a
smaller input (the array then still holds the first call's statistics)."""
import ctypes

import numpy as np
import pytest

from paper_2503_12964_amd import workloads as W
from tests import parity_utils as U

pytestmark = pytest.mark.gpu


def _binding():
    from paper_2503_12964_amd import binding
    binding.load_library()
    return binding


def _case(b, wl, gain=1.0):
    import torch
    inp = W.make_inputs(wl, gain_qk=gain)
    q, k, v, do = (U.to_device(inp[n]) for n in ("q", "k", "v", "dout"))
    out, lse = b.vfm_attn_fwd(q, k, v, wl.cu_seqlens, wl.scale)
    want = b.vfm_attn_bwd(q, k, v, out, lse, do, wl.cu_seqlens, wl.scale)
    got = tuple(torch.full_like(q, float("nan")) for _ in range(3))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    b.vfm_attn_bwd_noalloc(q, k, v, out, lse, do, wl.cu_seqlens, wl.scale, *got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert np.array_equal(U.to_bits(g), U.to_bits(w)), name
    return got


def test_noalloc_backward_matches_workspace_backward_twice():
    b = _binding()
    big = W.Workload("noalloc_big", ((3, 10, 10), (1, 1, 1), (1, 7, 11), (0, 1, 1), (3, 9, 19)), 3, 128,
                     (32, 48, 48), seed=21)
    small = W.Workload("noalloc_small", ((1, 5, 13), (1, 1, 2)), 2, 128, (32, 48, 48), seed=22)
    _case(b, big)
    _case(b, small)          # smaller input second: stale statistics of the first call lie behind it
    _case(b, W.Workload("noalloc_d64", ((2, 9, 15), (1, 5, 13)), 2, 64, (16, 24, 24), seed=23))


def test_noalloc_backward_rejects_sizes_beyond_its_scratch():
    b = _binding()
    lib = b.load_library()
    fake = ctypes.c_void_p(0x10000)     # never dereferenced: validation precedes any launch
    total, heads = 131072, 17           # 2,228,224 rows > VFM_NOALLOC_MAX_ROWS = 2,097,152
    cu = np.array([0, total], dtype=np.int32)
    st = lib.vfm_attn_bwd_noalloc(fake, fake, fake, fake, fake, fake,
                                  cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), 1, total, heads, 64, 0.125,
                                  fake, fake, fake, 0, None)
    assert st == 10
    assert b"VFM_NOALLOC_MAX_ROWS" in lib.vfm_strerror(st)
