"""Host-side checks of the C ABI: the library loads, exports what include/vfm.h declares,
and rejects bad arguments before launching anything (so no GPU is needed)."""
import ctypes
import os
import re
import subprocess
import sys

import numpy as np
import pytest

from paper_2503_12964_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2503_12964_amd.build import build_lib
        build_lib(verbose=False)
    return binding.load_library()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "vfm.h")).read()
    declared = set(re.findall(r"VFM_API\s+[\w\s\*]+?\b(vfm_\w+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_header_compiles_as_c_and_cxx(tmp_path):
    """include/vfm.h is a plain C header: it must compile on its own as C99 and as C++."""
    import shutil
    import subprocess
    header = os.path.join(ROOT, "include", "vfm.h")
    for compiler, std, suffix in (("gcc", "-std=c99", ".c"), ("g++", "-std=c++11", ".cc")):
        if shutil.which(compiler) is None:
            pytest.skip(f"{compiler} not available")
        src = tmp_path / ("use_vfm" + suffix)
        src.write_text(f'#include "{header}"\nint main(void) {{ return vfm_strerror(VFM_OK) == 0; }}\n')
        res = subprocess.run([compiler, std, "-Wall", "-Wextra", "-pedantic", "-fsyntax-only", str(src)],
                             capture_output=True, text=True)
        assert res.returncode == 0 and not res.stderr.strip(), res.stderr


def test_strerror_texts(lib):
    assert lib.vfm_strerror(0) == b"ok"
    texts = {lib.vfm_strerror(i) for i in range(11)}
    assert len(texts) == 11 and b"unknown status" not in texts
    assert lib.vfm_strerror(99) == b"unknown status"
    # no launch has failed in this process: the runtime's text for "success"
    assert lib.vfm_last_hip_error() == b"no error"


FAKE = ctypes.c_void_p(0x10000)      # never dereferenced: validation precedes any launch
ODD = ctypes.c_void_p(0x10008)
FAKE2 = ctypes.c_void_p(0x20000)


def _i32(a):
    arr = np.ascontiguousarray(np.asarray(a, dtype=np.int32))
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _fwd(lib, cu, total, heads=2, hd=128, scale=0.1, q=FAKE, out=FAKE, dt=0, n_seqs=None):
    arr, p = _i32(cu)
    n = len(cu) - 1 if n_seqs is None else n_seqs
    return lib.vfm_attn_fwd(q, FAKE, FAKE, p, n, total, heads, hd, scale, out, FAKE, dt, None)


def test_fwd_argument_errors(lib):
    assert _fwd(lib, [0, 8], 8, q=None) == 1
    assert _fwd(lib, [0, 8], 8, out=None) == 1
    assert _fwd(lib, [0, 8], 8, hd=96) == 2
    assert _fwd(lib, [0, 8], 8, heads=0) == 2
    assert _fwd(lib, [0, 8], 8, scale=0.0) == 2
    assert _fwd(lib, [0, 8], 8, scale=float("nan")) == 2
    assert _fwd(lib, [0] * 300, 0, n_seqs=299) == 0            # more clips than one table holds: legal
    assert _fwd(lib, [0] * 299 + [9], 8, n_seqs=299) == 3      # ... and still validated to the end
    assert _fwd(lib, [1, 8], 8) == 3
    assert _fwd(lib, [0, 5, 4, 8], 8) == 3
    assert _fwd(lib, [0, 7], 8) == 3
    assert _fwd(lib, [0, 8], 8, dt=1) == 6
    assert _fwd(lib, [0, 8], 8, q=ODD) == 9
    assert _fwd(lib, [0, 0, 0], 0) == 0                         # nothing to do is not an error


def test_rope_argument_errors(lib):
    def rope(thw, cu, total, dims=(32, 48, 48), hd=128, x=FAKE, theta=1e4, dt=0):
        a, pa = _i32(thw)
        b, pb = _i32(cu)
        return lib.vfm_rope3d(x, pa, pb, len(cu) - 1, total, 4, hd, dims[0], dims[1], dims[2], theta, 0, dt, None)
    assert rope([2, 2, 2], [0, 8], 8, x=None) == 1
    assert rope([2, 2, 2], [0, 8], 8, dims=(32, 48, 40)) == 5
    assert rope([2, 2, 2], [0, 8], 8, dims=(31, 49, 48)) == 5
    assert rope([2, 2, 2], [0, 8], 8, dims=(-2, 82, 48)) == 5
    assert rope([2, 2, 3], [0, 8], 8) == 4
    assert rope([2, 0, 4], [0, 8], 8) == 4
    assert rope([2, 2, 2], [0, 9], 8) == 3
    assert rope([2, 2, 2], [0, 8], 8, theta=0.0) == 2
    assert rope([2, 2, 2], [0, 8], 8, dt=1) == 6
    assert rope([2, 2, 2], [0, 8], 8, x=ODD) == 9
    assert rope([0, 0, 0], [0, 0], 0) == 0


def test_qknorm_rope_argument_errors(lib):
    a, thw = _i32([2, 2, 2])
    b, cu = _i32([0, 8])

    def fwd(x=FAKE, gain=FAKE, eps=1e-6, y=FAKE, dims=(32, 48, 48), total=8, dt=0):
        return lib.vfm_qknorm_rope3d(x, gain, eps, y, thw, cu, 1, total, 4, 128, dims[0], dims[1], dims[2],
                                     1e4, dt, None)

    def bwd(x=FAKE, gain=FAKE, eps=1e-6, dy=FAKE, dx=FAKE2, dgain=FAKE, total=8):
        return lib.vfm_qknorm_rope3d_bwd(x, gain, eps, dy, dx, dgain, thw, cu, 1, total, 4, 128, 32, 48, 48,
                                         1e4, 0, None)
    assert fwd(gain=None) == 1
    assert fwd(y=None) == 1
    assert fwd(eps=-1.0) == 2
    assert fwd(eps=float("nan")) == 2
    assert fwd(dims=(32, 48, 40)) == 5
    assert fwd(total=9) == 3
    assert fwd(dt=1) == 6
    assert fwd(x=ODD) == 9
    assert fwd(gain=ctypes.c_void_p(0x10002)) == 9
    assert bwd(dgain=None) == 1
    assert bwd(dx=FAKE) == 2                                    # dx must not be x
    assert bwd(dx=ODD) == 9
    assert bwd(eps=-1e-3) == 2
    assert bwd(total=7) == 3


def test_cross_attention_argument_errors(lib):
    def xf(cu_q, cu_kv, tq, tk, n=None, q=FAKE, dt=0, scale=0.1):
        a, pq = _i32(cu_q)
        b, pk = _i32(cu_kv)
        return lib.vfm_xattn_fwd(q, FAKE, FAKE, pq, pk, len(cu_q) - 1 if n is None else n, tq, tk, 2, 128, scale,
                                 FAKE, FAKE, dt, None)
    assert xf([0, 8], [0, 4], 8, 4, q=None) == 1
    assert xf([0, 8], [0, 4], 8, 5) == 3                        # cu_seqlens_kv does not end at total_kv
    assert xf([0, 4, 8], [0, 4, 4], 8, 4) == 3                  # queries without keys
    assert xf([0] * 130, [0] * 130, 0, 0) == 0                  # more sequences than one table holds: legal
    assert xf([0] * 129 + [8], [0] * 130, 8, 0) == 3            # queries without keys in the second run
    assert xf([0, 8], [0, 4], 8, 4, dt=1) == 6
    assert xf([0, 8], [0, 4], 8, 4, q=ODD) == 9
    assert xf([0, 8], [0, 4], 8, 4, scale=0.0) == 2
    assert xf([0, 0], [0, 0], 0, 0) == 0
    a, pq = _i32([0, 8])
    b, pk = _i32([0, 4])

    def xb(ws=FAKE, ws_bytes=1 << 30, dk=FAKE):
        return lib.vfm_xattn_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, pq, pk, 1, 8, 4, 2, 128, 0.1, FAKE, dk, FAKE,
                                 ws, ws_bytes, 0, None)
    assert xb(dk=None) == 1
    assert xb(ws=None) == 7
    assert xb(ws_bytes=16) == 7
    n = lib.vfm_xattn_bwd_workspace_size(8, 4, 2, 128)
    assert n % 256 == 0 and n >= lib.vfm_attn_bwd_workspace_size(8, 2, 128) + 2 * 4 * 2 * 128 * 4
    assert xb(ws_bytes=n - 1) == 7
    assert lib.vfm_xattn_bwd_workspace_size(8, 4, 2, 96) == 0


def test_temporal_attention_argument_errors(lib):
    def tf(thw, cu, total, q=FAKE, out=FAKE, dt=0, scale=0.1):
        a, pa = _i32(thw)
        b, pb = _i32(cu)
        return lib.vfm_tattn_fwd(q, FAKE, FAKE, pa, pb, len(cu) - 1, total, 2, 128, scale, out, dt, None)
    assert tf([2, 2, 2], [0, 8], 8, out=None) == 1
    assert tf([33, 1, 1], [0, 32], 32) == 4                     # grid and length disagree
    assert tf([2, 2, 3], [0, 8], 8) == 4
    assert tf([2, 2, 2], [0, 9], 8) == 3
    assert tf([2, 2, 2], [0, 8], 8, dt=1) == 6
    assert tf([2, 2, 2], [0, 8], 8, q=ODD) == 9
    assert tf([2, 2, 2], [0, 8], 8, scale=float("inf")) == 2
    assert tf([0, 0, 0], [0, 0], 0) == 0
    a, pa = _i32([2, 2, 2])
    b, pb = _i32([0, 8])
    assert lib.vfm_tattn_bwd(FAKE, FAKE, FAKE, FAKE, pa, pb, 1, 8, 2, 128, 0.1, FAKE, None, FAKE, 0, None) == 1
    assert lib.vfm_tattn_bwd(FAKE, FAKE, FAKE, FAKE, pa, pb, 1, 8, 2, 96, 0.1, FAKE, FAKE, FAKE, 0, None) == 2


def test_fp8_argument_errors(lib):
    arr, cu = _i32([0, 100, 100, 165])
    a, b, c, d = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    refs = (ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d))
    assert lib.vfm_fp8_pack_sizes(cu, 3, 165, 4, 128, *refs) == 0
    # units: ceil(100/64) + 0 + ceil(65/64) = 4
    assert a.value == 165 * 4 * 128 and b.value == 4 * 4 * 64 * 128 and c.value == b.value
    assert d.value == 768 + 4 * 4 * 4          # 660 q-row bytes padded to 768, then one word per (head, unit)
    assert lib.vfm_fp8_pack_sizes(cu, 3, 166, 4, 128, *refs) == 3
    assert lib.vfm_fp8_pack_sizes(cu, 3, 165, 4, 96, *refs) == 2
    assert lib.vfm_fp8_pack_sizes(cu, 3, 165, 4, 128, None, *refs[1:]) == 1
    many, pm = _i32([0] * 300)
    assert lib.vfm_fp8_pack_sizes(pm, 299, 0, 4, 128, *refs) == 0            # more clips than one table holds: legal

    def pack(q=FAKE, scale=0.09, q8=FAKE, scales=FAKE, dt=0):
        return lib.vfm_fp8_pack(q, FAKE, FAKE, cu, 3, 165, 4, 128, scale, q8, FAKE, FAKE, scales, dt, None)
    assert pack(q=None) == 1
    assert pack(scales=None) == 1
    assert pack(scale=0.0) == 2
    assert pack(scale=float("inf")) == 2
    assert pack(dt=1) == 6
    assert pack(q8=ODD) == 9

    def fwd(q8=FAKE, scales=FAKE, lse=FAKE):
        return lib.vfm_attn_fwd_fp8(q8, FAKE, FAKE, scales, cu, 3, 165, 4, 128, FAKE, lse, None)
    assert fwd(lse=None) == 1
    assert fwd(scales=None) == 1
    assert fwd(q8=ODD) == 9


def test_forward_tile_rows_rule(lib):
    def rows(cu, hd, run=0):
        arr, p = _i32(cu)
        r = ctypes.c_int(-1)
        st = lib.vfm_attn_fwd_tile_rows(p, len(cu) - 1, cu[-1], hd, run, ctypes.byref(r))
        return st, r.value
    assert rows([0, 56320], 128) == (0, 256)
    assert rows([0, 1024, 2048], 128) == (0, 128)               # longest clip <= 1,024 tokens
    assert rows([0, 1025], 128) == (0, 256)
    assert rows([0, 56320], 64) == (0, 128)
    cu = [0] + [2000] * 256 + [2100]                            # run 0 holds the long clip, run 1 a short one
    assert rows(cu, 128, 0) == (0, 256) and rows(cu, 128, 1) == (0, 128)
    assert rows(cu, 128, 2)[0] == 2                             # no such run
    assert rows([0, 8], 96)[0] == 2
    assert rows([0, 8, 7], 128)[0] == 3


def test_tensors_beyond_32bit_byte_offsets_are_rejected(lib):
    # 131072 tokens x 128 heads x 128 x 2 bytes = 4 GiB: the kernels address tensors with 32-bit byte offsets
    arr, p = _i32([0, 131072])
    assert lib.vfm_attn_fwd(FAKE, FAKE, FAKE, p, 1, 131072, 128, 128, 0.1, FAKE, FAKE, 0, None) == 2
    assert lib.vfm_attn_bwd_workspace_size(131072, 128, 128) == 0


def test_bwd_argument_errors_and_workspace(lib):
    size = lib.vfm_attn_bwd_workspace_size
    assert size(0, 2, 128) == 0 or size(0, 2, 128) % 256 == 0
    assert size(10, 2, 96) == 0
    n = size(1000, 4, 128)
    assert n >= 1000 * 4 * 4 and n % 256 == 0
    arr, p = _i32([0, 8])

    def bwd(ws=FAKE, ws_bytes=1 << 30, dq=FAKE, cu=p, total=8):
        return lib.vfm_attn_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, cu, 1, total, 2, 128, 0.1, dq, FAKE, FAKE,
                                ws, ws_bytes, 0, None)
    assert bwd(dq=None) == 1
    assert bwd(ws=None) == 7
    assert bwd(ws_bytes=16) == 7
    assert bwd(ws=ctypes.c_void_p(0x10010)) == 7                # not 256-byte aligned
    assert bwd(total=9) == 3


def test_library_shares_pytorchs_hip_runtime():
    # A process that loads the library before it ever imported torch must still end up with a
    # single HIP runtime (a second copy of the runtime finds no device on a GPU machine).
    code = ("from paper_2503_12964_amd import binding\n"
            "binding.load_library()\n"
            "import torch\n"
            "libs = {l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l}\n"
            "print(len(libs))\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-1000:]
    assert r.stdout.strip().splitlines()[-1] == "1", r.stdout


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "libvfm.so"))
