// Token -> grid position -> rotation angles, shared by the RoPE kernels (gfx950 only).
#pragma once

#include <math.h>

#include "vfm_common.h"

namespace vfm {

struct RopeFreq {
  double inv_freq[64];    // per pair index p = element/2: theta^(-2i/d_axis)
  unsigned char axis[64]; // 0 = t, 1 = h, 2 = w
};

// Host: per-pair inverse frequencies and axis of each pair for a (d_t, d_h, d_w) split.
inline RopeFreq make_rope_freq(int dim_t, int dim_h, int dim_w, float theta) {
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
  return fr;
}

// (cos, sin) of the four adjacent pairs in 16-byte chunk `chunk` of token `tok`'s head
// vectors.  The angle is formed and reduced to [-pi, pi] in fp64 (a handful of operations
// per token, reused for every head), so the rotation stays accurate to fp32 rounding
// however large the grid position is.  negate != 0 gives the transpose rotation.
__device__ __forceinline__ void rope_cos_sin(const RopeTable& tab, const RopeFreq& fr, int tok,
                                             int chunk, int negate, float (&cs)[4], float (&sn)[4]) {
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
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int p = chunk * 4 + e;
    const int ax = fr.axis[p];
    const double pa = (double)(ax == 0 ? pos[0] : (ax == 1 ? pos[1] : pos[2]));
    double ang = pa * fr.inv_freq[p];
    ang -= 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
    float s, c;
    sincosf((float)ang, &s, &c);
    cs[e] = c;
    sn[e] = negate ? -s : s;
  }
}

// bf16 pair packed in a 32-bit word <-> two floats
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 y = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(y, bf16x2));
}

}  // namespace vfm
