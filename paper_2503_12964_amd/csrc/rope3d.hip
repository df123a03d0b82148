// 3D rotary position embedding, in place, HBM-bound.
//
// One group of D/8 lanes owns one token; lane c of the group owns the 16-byte
// chunk c of every head vector of that token (four adjacent pairs).  The four
// (cos, sin) values a lane needs depend on the token and on c only, so they are
// computed once (angle reduced in fp64, then sincosf) and reused for all
// heads.  A wavefront therefore moves 256-byte contiguous head rows; every byte
// of x is read once and written once.
#include "rope_common.h"

namespace vfm {

template <int D>
__global__ __launch_bounds__(256) void rope3d_kernel(u32x4* __restrict__ x, const RopeTable tab,
                                                     const RopeFreq fr, int tok0, int tok_end,
                                                     int n_heads, int inverse) {
  // tokens [tok0, tok_end): the clips of tab (a call with more clips than a table holds is cut
  // into consecutive launches over runs of clips)
  constexpr int kLanesPerTok = D / 8;
  constexpr int kTokPerBlock = 256 / kLanesPerTok;
  const int tok = tok0 + blockIdx.x * kTokPerBlock + threadIdx.x / kLanesPerTok;
  const int chunk = threadIdx.x % kLanesPerTok;
  if (tok >= tok_end) return;

  float cs[4], sn[4];
  rope_cos_sin(tab, fr, tok, chunk, inverse, cs, sn);

  u32x4* row = x + ((size_t)tok * n_heads) * kLanesPerTok + chunk;
  constexpr int kUnroll = 4;
  int h = 0;
  for (; h + kUnroll <= n_heads; h += kUnroll) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(row + (size_t)(h + u) * kLanesPerTok);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      u32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x0 = __builtin_bit_cast(float, v[u][e] << 16);
        const float x1 = __builtin_bit_cast(float, v[u][e] & 0xffff0000u);
        f32x2 y;
        y[0] = x0 * cs[e] - x1 * sn[e];
        y[1] = x0 * sn[e] + x1 * cs[e];
        o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(y, bf16x2));
      }
      __builtin_nontemporal_store(o, row + (size_t)(h + u) * kLanesPerTok);
    }
  }
  for (; h < n_heads; ++h) {
    const u32x4 v = row[(size_t)h * kLanesPerTok];
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x0 = __builtin_bit_cast(float, v[e] << 16);
      const float x1 = __builtin_bit_cast(float, v[e] & 0xffff0000u);
      f32x2 y;
      y[0] = x0 * cs[e] - x1 * sn[e];
      y[1] = x0 * sn[e] + x1 * cs[e];
      o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(y, bf16x2));
    }
    row[(size_t)h * kLanesPerTok] = o;
  }
}

hipError_t launch_rope3d(void* x, const RopeTable& tab, int n_heads, int head_dim,
                         int dim_t, int dim_h, int dim_w, float theta, int inverse,
                         hipStream_t stream) {
  const RopeFreq fr = make_rope_freq(dim_t, dim_h, dim_w, theta);
  const int tok0 = tab.cu[0], tok_end = tab.cu[tab.n], count = tok_end - tok0;
  if (count == 0) return hipSuccess;
  if (head_dim == 128)
    return launch(rope3d_kernel<128>, dim3((count + 15) / 16), dim3(256), 0, stream, (u32x4*)x, tab, fr, tok0,
                  tok_end, n_heads, inverse);
  return launch(rope3d_kernel<64>, dim3((count + 31) / 32), dim3(256), 0, stream, (u32x4*)x, tab, fr, tok0,
                tok_end, n_heads, inverse);
}

}  // namespace vfm
