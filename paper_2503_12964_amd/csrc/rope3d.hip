// 3D rotary position embedding, in place, HBM-bound.
//
// One group of D/8 lanes owns one token; lane c of the group owns the 16-byte
// chunk c of every head vector of that token (four adjacent pairs).  The four
// (cos, sin) values a lane needs depend on the token and on c only, so they are
// computed once (angle reduced in fp64, then sincosf) and reused for all
// heads.  A wavefront therefore moves 256-byte contiguous head rows; every byte
// of x is read once and written once.
#include "vfm_common.h"

namespace vfm {

struct RopeFreq {
  double inv_freq[64];    // per pair index p = element/2: theta^(-2i/d_axis)
  unsigned char axis[64]; // 0 = t, 1 = h, 2 = w
};

template <int D>
__global__ __launch_bounds__(256) void rope3d_kernel(u32x4* __restrict__ x, const RopeTable tab,
                                                     const RopeFreq fr, int total, int n_heads,
                                                     int inverse) {
  constexpr int kLanesPerTok = D / 8;
  constexpr int kTokPerBlock = 256 / kLanesPerTok;
  const int tok = blockIdx.x * kTokPerBlock + threadIdx.x / kLanesPerTok;
  const int chunk = threadIdx.x % kLanesPerTok;
  if (tok >= total) return;

  // clip of this token: last s with cu[s] <= tok (skips empty clips)
  int lo = 0, hi = tab.n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tab.cu[mid] <= tok) lo = mid; else hi = mid;
  }
  const int r = tok - tab.cu[lo];
  const int hw = tab.hw[lo], w = tab.w[lo];
  int pos[3];
  pos[0] = r / hw;
  const int rem = r - pos[0] * hw;
  pos[1] = rem / w;
  pos[2] = rem - pos[1] * w;

  float cs[4], sn[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int p = chunk * 4 + e;
    const int ax = fr.axis[p];
    // The angle is formed and reduced to [-pi, pi] in fp64 (a handful of operations per
    // token, reused for every head), so the rotation stays accurate to fp32 rounding
    // however large the grid position is.
    const double pa = (double)(ax == 0 ? pos[0] : (ax == 1 ? pos[1] : pos[2]));
    double ang = pa * fr.inv_freq[p];
    ang -= 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
    float s, c;
    sincosf((float)ang, &s, &c);
    cs[e] = c;
    sn[e] = inverse ? -s : s;
  }

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

hipError_t launch_rope3d(void* x, const RopeTable& tab, int total, int n_heads, int head_dim,
                         int dim_t, int dim_h, int dim_w, float theta, int inverse,
                         hipStream_t stream) {
  RopeFreq fr;
  const int dims[3] = {dim_t, dim_h, dim_w};
  int p = 0;
  for (int ax = 0; ax < 3; ++ax) {
    for (int i = 0; i < dims[ax] / 2; ++i, ++p) {
      fr.inv_freq[p] = pow((double)theta, -2.0 * (double)i / (double)dims[ax]);
      fr.axis[p] = (unsigned char)ax;
    }
  }
  for (; p < 64; ++p) { fr.inv_freq[p] = 0.0; fr.axis[p] = 0; }
  if (total == 0) return hipSuccess;
  if (head_dim == 128) {
    const int grid = (total + 15) / 16;
    rope3d_kernel<128><<<grid, 256, 0, stream>>>((u32x4*)x, tab, fr, total, n_heads, inverse);
  } else {
    const int grid = (total + 31) / 32;
    rope3d_kernel<64><<<grid, 256, 0, stream>>>((u32x4*)x, tab, fr, total, n_heads, inverse);
  }
  return hipGetLastError();
}

}  // namespace vfm
