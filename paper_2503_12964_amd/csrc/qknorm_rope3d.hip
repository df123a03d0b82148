// Per-head RMS normalisation with a learned gain, fused with 3D rotary position embedding
// (forward and backward), HBM-bound.
//
//   forward :  r = rsqrt(mean_d x_d^2 + eps),  z = x r g,  y = R z
//   backward:  dz = R^T dy,  dgain += dz (x r),  dn = dz g,
//              dx = r (dn - (x r) mean_d(dn_d x_d r))
//
// Same work split as the plain RoPE kernel: a group of D/8 lanes owns one token, lane c of
// the group owns the 16-byte chunk c of every head vector of that token, and the four
// (cos, sin) pairs of that chunk are computed once per token and reused for all heads.
// The per-(token, head) sums over head_dim are reductions over the D/8 lanes of a group,
// done with DPP lane permutes inside one 16-lane row (no LDS, no extra pass over memory),
// so every byte is still read once and written once.  The backward recomputes r from x
// instead of reading a saved statistic.  dgain is summed per lane over the heads and tokens
// a workgroup visits, reduced across the workgroup in LDS, and added to memory with one
// fp32 atomic per workgroup and element (its summation order, hence its last bits, may
// differ between runs).
#include "rope_common.h"

namespace vfm {

namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int o = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
  return v + __builtin_bit_cast(float, o);
}

// Sum over the LANES (8 or 16) consecutive lanes of a token group; every lane gets the
// total.  Groups are aligned to their size, so all permutes stay inside the group:
// xor 1 and xor 2 within quads, then mirror within 8 lanes, then mirror within 16.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
  v = dpp_add<0x141>(v);   // row_half_mirror
  if constexpr (LANES == 16) v = dpp_add<0x140>(v);   // row_mirror
  return v;
}

__device__ __forceinline__ void unpack8(const u32x4& v, float (&f)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = bf16_lo(v[e]);
    f[2 * e + 1] = bf16_hi(v[e]);
  }
}

}  // namespace

template <int D>
__global__ __launch_bounds__(256) void qknorm_rope3d_kernel(const u32x4* x, u32x4* y,
                                                            const float* __restrict__ gain, float eps,
                                                            const RopeTable tab, const RopeFreq fr,
                                                            int tok0, int tok_end, int n_heads) {
  constexpr int kLanesPerTok = D / 8;
  constexpr int kTokPerBlock = 256 / kLanesPerTok;
  const int tok = tok0 + blockIdx.x * kTokPerBlock + threadIdx.x / kLanesPerTok;   // the clips of tab
  const int chunk = threadIdx.x % kLanesPerTok;
  if (tok >= tok_end) return;   // whole groups leave together

  float cs[4], sn[4];
  rope_cos_sin(tab, fr, tok, chunk, 0, cs, sn);
  float g[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) g[e] = gain[chunk * 8 + e];

  const size_t base = ((size_t)tok * n_heads) * kLanesPerTok + chunk;
  constexpr int kUnroll = 4;
  for (int h0 = 0; h0 < n_heads; h0 += kUnroll) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (h0 + u < n_heads) v[u] = __builtin_nontemporal_load(x + base + (size_t)(h0 + u) * kLanesPerTok);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      if (h0 + u >= n_heads) break;     // uniform over the workgroup
      float f[8];
      unpack8(v[u], f);
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = __builtin_fmaf(f[e], f[e], ss);
      ss = group_sum<kLanesPerTok>(ss);
      const float r = 1.0f / __builtin_sqrtf(ss * (1.0f / D) + eps);
      u32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float z0 = f[2 * e] * r * g[2 * e];
        const float z1 = f[2 * e + 1] * r * g[2 * e + 1];
        o[e] = pack_bf16x2(z0 * cs[e] - z1 * sn[e], z0 * sn[e] + z1 * cs[e]);
      }
      __builtin_nontemporal_store(o, y + base + (size_t)(h0 + u) * kLanesPerTok);
    }
  }
}

__global__ void zero_f32_kernel(float* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

template <int D>
__global__ __launch_bounds__(256) void qknorm_rope3d_bwd_kernel(const u32x4* __restrict__ x,
                                                                const u32x4* dy, u32x4* dx,
                                                                const float* __restrict__ gain, float eps,
                                                                float* __restrict__ dgain,
                                                                const RopeTable tab, const RopeFreq fr,
                                                                int tok0, int tok_end, int n_heads) {
  constexpr int kLanesPerTok = D / 8;
  constexpr int kTokPerBlock = 256 / kLanesPerTok;
  __shared__ float red[kTokPerBlock][D];
  const int group = threadIdx.x / kLanesPerTok;
  const int chunk = threadIdx.x % kLanesPerTok;

  float g[8], dg[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { g[e] = gain[chunk * 8 + e]; dg[e] = 0.f; }

  // whole groups iterate together; nobody returns before the barrier below
  for (int tok = tok0 + blockIdx.x * kTokPerBlock + group; tok < tok_end; tok += gridDim.x * kTokPerBlock) {
    float cs[4], sn[4];
    rope_cos_sin(tab, fr, tok, chunk, 1, cs, sn);   // transpose rotation
    const size_t base = ((size_t)tok * n_heads) * kLanesPerTok + chunk;
    constexpr int kUnroll = 2;
    for (int h0 = 0; h0 < n_heads; h0 += kUnroll) {
      u32x4 xv[kUnroll], gv[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        if (h0 + u < n_heads) {
          xv[u] = __builtin_nontemporal_load(x + base + (size_t)(h0 + u) * kLanesPerTok);
          gv[u] = __builtin_nontemporal_load(dy + base + (size_t)(h0 + u) * kLanesPerTok);
        }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        if (h0 + u >= n_heads) break;   // uniform over the workgroup
        float f[8], d[8];
        unpack8(xv[u], f);
        unpack8(gv[u], d);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = __builtin_fmaf(f[e], f[e], ss);
        ss = group_sum<kLanesPerTok>(ss);
        const float r = 1.0f / __builtin_sqrtf(ss * (1.0f / D) + eps);
        float n[8], dn[8];
        float t = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float dz0 = d[2 * e] * cs[e] - d[2 * e + 1] * sn[e];
          const float dz1 = d[2 * e] * sn[e] + d[2 * e + 1] * cs[e];
          n[2 * e] = f[2 * e] * r;
          n[2 * e + 1] = f[2 * e + 1] * r;
          dg[2 * e] = __builtin_fmaf(dz0, n[2 * e], dg[2 * e]);
          dg[2 * e + 1] = __builtin_fmaf(dz1, n[2 * e + 1], dg[2 * e + 1]);
          dn[2 * e] = dz0 * g[2 * e];
          dn[2 * e + 1] = dz1 * g[2 * e + 1];
          t = __builtin_fmaf(dn[2 * e], n[2 * e], t);
          t = __builtin_fmaf(dn[2 * e + 1], n[2 * e + 1], t);
        }
        t = group_sum<kLanesPerTok>(t) * (1.0f / D);
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          o[e] = pack_bf16x2(r * (dn[2 * e] - n[2 * e] * t), r * (dn[2 * e + 1] - n[2 * e + 1] * t));
        __builtin_nontemporal_store(o, dx + base + (size_t)(h0 + u) * kLanesPerTok);
      }
    }
  }

#pragma unroll
  for (int e = 0; e < 8; ++e) red[group][chunk * 8 + e] = dg[e];
  __syncthreads();
  for (int d = threadIdx.x; d < D; d += 256) {
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < kTokPerBlock; ++t) s += red[t][d];
    atomicAdd(dgain + d, s);
  }
}

hipError_t launch_qknorm_rope3d(const void* x, void* y, const float* gain, float eps,
                                const RopeTable& tab, int n_heads, int head_dim,
                                int dim_t, int dim_h, int dim_w, float theta, hipStream_t stream) {
  const int tok0 = tab.cu[0], tok_end = tab.cu[tab.n], count = tok_end - tok0;
  if (count == 0) return hipSuccess;
  const RopeFreq fr = make_rope_freq(dim_t, dim_h, dim_w, theta);
  if (head_dim == 128)
    return launch(qknorm_rope3d_kernel<128>, dim3((count + 15) / 16), dim3(256), 0, stream, (const u32x4*)x,
                  (u32x4*)y, gain, eps, tab, fr, tok0, tok_end, n_heads);
  return launch(qknorm_rope3d_kernel<64>, dim3((count + 31) / 32), dim3(256), 0, stream, (const u32x4*)x,
                (u32x4*)y, gain, eps, tab, fr, tok0, tok_end, n_heads);
}

hipError_t launch_zero_f32(float* p, int n, hipStream_t stream) {
  return launch(zero_f32_kernel, dim3((n + 127) / 128), dim3(128), 0, stream, p, n);
}

// dgain is accumulated into (zeroed by the caller with launch_zero_f32 before the first run of clips)
hipError_t launch_qknorm_rope3d_bwd(const void* x, const void* dy, void* dx, const float* gain,
                                    float eps, float* dgain, const RopeTable& tab,
                                    int n_heads, int head_dim, int dim_t, int dim_h, int dim_w,
                                    float theta, hipStream_t stream) {
  const int tok0 = tab.cu[0], tok_end = tab.cu[tab.n], count = tok_end - tok0;
  if (count == 0) return hipSuccess;
  const RopeFreq fr = make_rope_freq(dim_t, dim_h, dim_w, theta);
  constexpr int kMaxGrid = 4096;   // bounds the number of atomics; more tokens loop
  if (head_dim == 128) {
    const int grid = min((count + 15) / 16, kMaxGrid);
    return launch(qknorm_rope3d_bwd_kernel<128>, dim3(grid), dim3(256), 0, stream, (const u32x4*)x,
                  (const u32x4*)dy, (u32x4*)dx, gain, eps, dgain, tab, fr, tok0, tok_end, n_heads);
  }
  const int grid = min((count + 31) / 32, kMaxGrid);
  return launch(qknorm_rope3d_bwd_kernel<64>, dim3(grid), dim3(256), 0, stream, (const u32x4*)x,
                (const u32x4*)dy, (u32x4*)dx, gain, eps, dgain, tab, fr, tok0, tok_end, n_heads);
}

}  // namespace vfm
