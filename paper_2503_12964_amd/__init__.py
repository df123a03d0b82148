"""MI355X-native packed 3D-RoPE attention (forward and backward) behind libvfm.so.

`binding` holds the ctypes wrappers over the C ABI declared in include/vfm.h;
`workloads` holds the seeded synthetic inputs; `build` compiles the library.
Nothing is loaded at import time; the first call into `binding` loads
libvfm.so and raises if it has not been built.
"""
from .binding import (VfmError, load_library, strerror, vfm_attn_bwd,  # noqa: F401
                      vfm_attn_fwd_fp8, vfm_fp8_pack, vfm_fp8_pack_sizes,
                      vfm_attn_bwd_workspace_size, vfm_attn_fwd, vfm_qknorm_rope3d,
                      vfm_qknorm_rope3d_bwd, vfm_rope3d, vfm_tattn_bwd, vfm_tattn_fwd,
                      vfm_xattn_bwd, vfm_xattn_bwd_workspace_size, vfm_xattn_fwd)
