// Temporal attention for gfx950: one sequence per (clip, pixel) made of that pixel's token
// in every latent frame (T rows, H*W tokens apart in the packed buffer), per head.
// HBM-bound up to 32 frames: the whole problem of one (pixel, head) is a 16 x 16 score tile (a
// 32 x 32 one, further down, when a clip has more than 16 frames).  Clips with more than 32
// frames are walked in 32-row blocks by the kernels at the end of the file.
//
// One wavefront owns one (pixel, head).  It gathers the T rows of q, k, v (and dout) into a
// wave-private LDS tile with direct global->LDS loads (16-byte chunks, 256-byte rows, the same
// XOR swizzle as the other attention kernels), and needs no workgroup barrier at all.
//   S^T = K Q^T            v_mfma_f32_16x16x32_bf16, A = K rows, B = Q rows
// leaves lane l with query i = l % 16 and keys j = 4*(l/16) + r in its four registers, so the
// softmax is a 4-register reduction plus two lane exchanges (xor 16, xor 32), and the
// normalised bf16 P^T registers are the B operand of
//   O^T = V^T P^T          v_mfma_f32_16x16x16_bf16, A = V^T through transposing LDS reads.
// The backward recomputes the softmax (no saved statistics; Delta_i = sum_j P_ij dP_ij) and
// needs P and dS in both orientations -- lane = query for dQ, lane = key for dK and dV -- which
// it gets by issuing the score MFMAs twice with the operands swapped.
// Rows past T are clamped copies of row T-1: as keys they are masked, as queries their
// results are not stored and their P is zeroed where it would be summed into dK/dV.
#include <algorithm>

#include "vfm_common.h"

namespace vfm {

namespace {

constexpr int kTRows = 16;       // rows of a temporal tile = largest T served
constexpr int kTWaves = 4;
constexpr float kLog2eT = 1.4426950408889634f;

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <int D>
struct TCfg {
  static constexpr int kTileBytes = kTRows * D * 2;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kLoadsPerTile = kTRows * kChunksPerRow / 64;
};

__device__ __forceinline__ f32x4v mfma16x32(bf16x8 a, bf16x8 b, f32x4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4v mfma16x16(bf16x4 a, bf16x4 b, f32x4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x4 lds_tr4(const char* base, int off) {
  return __builtin_bit_cast(bf16x4, lds_read_tr(base, off));
}

// Which (clip, pixel, head) this wavefront owns.  Returns false past the end.
struct TUnit {
  int head, first_row, hw, T;   // rows of the sequence: first_row + t*hw, t < T
};
__device__ __forceinline__ bool temporal_unit(const TemporalTable& tab, int n_heads, TUnit& u) {
  const long long unit = (long long)blockIdx.x * kTWaves + (threadIdx.x >> 6);
  const long long n_units = (long long)tab.pix_cu[tab.n] * n_heads;
  if (unit >= n_units) return false;
  u.head = (int)(unit % n_heads);
  const int pp = (int)(unit / n_heads);
  int lo = 0, hi = tab.n;            // last clip s with pix_cu[s] <= pp (skips empty clips)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tab.pix_cu[mid] <= pp) lo = mid; else hi = mid;
  }
  u.hw = tab.hw[lo];
  u.first_row = tab.cu[lo] + (pp - tab.pix_cu[lo]);
  u.T = (tab.cu[lo + 1] - tab.cu[lo]) / u.hw;
  return true;
}

// Gather the sequence's rows of one tensor into a swizzled [16][D] LDS tile.
template <int D>
__device__ __forceinline__ void gather_tile(const __bf16* base, const TUnit& u, uint32_t row_bytes,
                                            uint32_t lds_tile, int lane) {
  using Cfg = TCfg<D>;
#pragma unroll
  for (int x = 0; x < Cfg::kLoadsPerTile; ++x) {
    const int p = x * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    const int chunk = (p % Cfg::kChunksPerRow) ^ swz<D>(r);
    const uint32_t off = (uint32_t)(u.first_row + min(r, u.T - 1) * u.hw) * row_bytes +
                         (uint32_t)(u.head * D * 2 + chunk * 16);
    lds_dma16(base, off, lds_tile + x * 1024);
  }
}

// Row operands of a tile for the 16x16x32 MFMA: lane l holds row l%16, columns ks*32 + 8*(l/16)..+7.
template <int D>
__device__ __forceinline__ void read_rows(const char* tile, int lane, bf16x8 (&f)[D / 32]) {
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) f[ks] = lds_read_b128(tile, tile_off<D>(lane & 15, ks * 32 + 8 * (lane >> 4)));
}

// Transposed operand for the 16x16x16 MFMA: lane l gets X[4*(l/16) + r][db*16 + l%16], r < 4.
template <int D>
__device__ __forceinline__ bf16x4 read_tr(const char* tile, int lane, int db) {
  return lds_tr4(tile, tile_off<D>(4 * (lane >> 4) + ((lane & 15) >> 2), db * 16 + 4 * (lane & 3)));
}

__device__ __forceinline__ float quad_group_max(float x) {   // over lanes l, l^16, l^32, l^48
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float quad_group_sum(float x) {
  x += __shfl_xor(x, 16);
  return x + __shfl_xor(x, 32);
}

// Store a 16x16x16 result tile C[d = db*16 + 4*(l/16) + r][token = l%16] as 4 bf16 of row `token`.
template <int D>
__device__ __forceinline__ void store_tile(__bf16* base, const TUnit& u, size_t row_stride, int lane,
                                           int db, f32x4v c, float mul) {
  if ((lane & 15) < u.T) {
    const size_t row = (size_t)(u.first_row + (lane & 15) * u.hw);
    f32x4 o = {c[0] * mul, c[1] * mul, c[2] * mul, c[3] * mul};
    *reinterpret_cast<bf16x4*>(base + row * row_stride + (size_t)u.head * D + db * 16 + 4 * (lane >> 4)) =
        to_bf16x4(o);
  }
}

}  // namespace

template <int D>
__global__ __launch_bounds__(kTWaves * 64) void tattn_fwd_kernel(const __bf16* __restrict__ q,
                                                                 const __bf16* __restrict__ k,
                                                                 const __bf16* __restrict__ v,
                                                                 __bf16* __restrict__ out,
                                                                 const TemporalTable tab, int n_heads,
                                                                 float scale_log2) {
  using Cfg = TCfg<D>;
  constexpr int TB = Cfg::kTileBytes;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  TUnit u;
  if (!temporal_unit(tab, n_heads, u)) return;   // whole wavefronts leave; there are no barriers
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const size_t row_stride = (size_t)n_heads * D;
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  char* mine = smem + wave * 3 * TB;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(mine));
  gather_tile<D>(q, u, row_bytes, lds0, lane);
  gather_tile<D>(k, u, row_bytes, lds0 + TB, lane);
  gather_tile<D>(v, u, row_bytes, lds0 + 2 * TB, lane);
  wait_vmcnt<0>();

  bf16x8 qf[D / 32], kf[D / 32];
  read_rows<D>(mine, lane, qf);
  read_rows<D>(mine + TB, lane, kf);
  f32x4v st = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) st = mfma16x32(kf[ks], qf[ks], st);
  // lane: query l%16; register r: key 4*(l/16) + r
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    if (4 * (lane >> 4) + r >= u.T) st[r] = -INFINITY;
    mx = fmaxf(mx, st[r]);
  }
  const float m2 = quad_group_max(mx) * scale_log2;
  f32x4 p;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    p[r] = fast_exp2(st[r] * scale_log2 - m2);
    sum += p[r];
  }
  const float inv = 1.0f / quad_group_sum(sum);
#pragma unroll
  for (int r = 0; r < 4; ++r) p[r] *= inv;
  const bf16x4 pb = to_bf16x4(p);
  const f32x4v zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int db = 0; db < D / 16; ++db) {
    const f32x4v o = mfma16x16(read_tr<D>(mine + 2 * TB, lane, db), pb, zero);
    store_tile<D>(out, u, row_stride, lane, db, o, 1.0f);
  }
}

template <int D>
__global__ __launch_bounds__(kTWaves * 64) void tattn_bwd_kernel(const __bf16* __restrict__ q,
                                                                 const __bf16* __restrict__ k,
                                                                 const __bf16* __restrict__ v,
                                                                 const __bf16* __restrict__ dout,
                                                                 __bf16* __restrict__ dq,
                                                                 __bf16* __restrict__ dk,
                                                                 __bf16* __restrict__ dv,
                                                                 const TemporalTable tab, int n_heads,
                                                                 float scale, float scale_log2) {
  using Cfg = TCfg<D>;
  constexpr int TB = Cfg::kTileBytes;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  TUnit u;
  if (!temporal_unit(tab, n_heads, u)) return;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const size_t row_stride = (size_t)n_heads * D;
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  char* qt = smem + wave * 4 * TB;
  char* kt = qt + TB;
  char* vt = qt + 2 * TB;
  char* dot = qt + 3 * TB;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(qt));
  gather_tile<D>(q, u, row_bytes, lds0, lane);
  gather_tile<D>(k, u, row_bytes, lds0 + TB, lane);
  gather_tile<D>(v, u, row_bytes, lds0 + 2 * TB, lane);
  gather_tile<D>(dout, u, row_bytes, lds0 + 3 * TB, lane);
  wait_vmcnt<0>();

  bf16x8 qf[D / 32], kf[D / 32], vf[D / 32], df[D / 32];
  read_rows<D>(qt, lane, qf);
  read_rows<D>(kt, lane, kf);
  read_rows<D>(vt, lane, vf);
  read_rows<D>(dot, lane, df);
  // "A": lane = query, registers = keys (S^T, dP^T);  "B": lane = key, registers = queries (S, dP)
  f32x4v sA = {0.f, 0.f, 0.f, 0.f}, sB = sA, dpA = sA, dpB = sA;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    sA = mfma16x32(kf[ks], qf[ks], sA);
    sB = mfma16x32(qf[ks], kf[ks], sB);
    dpA = mfma16x32(vf[ks], df[ks], dpA);
    dpB = mfma16x32(df[ks], vf[ks], dpB);
  }
  const int base_r = 4 * (lane >> 4);
  // softmax statistics per query, in orientation A
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    if (base_r + r >= u.T) sA[r] = -INFINITY;
    mx = fmaxf(mx, sA[r]);
  }
  const float m2 = quad_group_max(mx) * scale_log2;
  float pA[4], sum = 0.f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    pA[r] = fast_exp2(sA[r] * scale_log2 - m2);
    sum += pA[r];
  }
  sum = quad_group_sum(sum);
  const float lse2 = m2 + __log2f(sum);      // P = exp2(s*scale_log2 - lse2)
  const float inv = 1.0f / sum;
  float dl = 0.f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    pA[r] *= inv;
    dl += pA[r] * dpA[r];
  }
  const float delta = quad_group_sum(dl);    // Delta_i = sum_j P_ij dP_ij
  f32x4 dsA;
#pragma unroll
  for (int r = 0; r < 4; ++r) dsA[r] = pA[r] * (dpA[r] - delta);
  const bf16x4 dsAb = to_bf16x4(dsA);
  // orientation B: register r belongs to query base_r + r, whose statistics lane base_r + r holds
  f32x4 pB, dsB;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float l2 = __shfl(lse2, base_r + r);
    const float dd = __shfl(delta, base_r + r);
    const float pv = (base_r + r < u.T) ? fast_exp2(sB[r] * scale_log2 - l2) : 0.f;   // padded queries add nothing
    pB[r] = pv;
    dsB[r] = pv * (dpB[r] - dd);
  }
  const bf16x4 pBb = to_bf16x4(pB), dsBb = to_bf16x4(dsB);
  const f32x4v zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int db = 0; db < D / 16; ++db) {
    // dV^T[d, j] = sum_i dO[i, d] P[i, j];  dK^T[d, j] = scale sum_i Q[i, d] dS[i, j]
    store_tile<D>(dv, u, row_stride, lane, db, mfma16x16(read_tr<D>(dot, lane, db), pBb, zero), 1.0f);
    store_tile<D>(dk, u, row_stride, lane, db, mfma16x16(read_tr<D>(qt, lane, db), dsBb, zero), scale);
    // dQ^T[d, i] = scale sum_j K[j, d] dS^T[j, i]
    store_tile<D>(dq, u, row_stride, lane, db, mfma16x16(read_tr<D>(kt, lane, db), dsAb, zero), scale);
  }
}

// ---------------------------------------------------------------- 17..32 frames
// The same scheme on a 32 x 32 score tile with the 32x32x16 MFMA (lane layouts as in the packed
// attention kernels: an operand lane holds row l%32, columns ks*16 + 8*(l/32)..+7; an accumulator
// lane holds column l%32, rows 8*(r/4) + 4*(l/32) + r%4 in its sixteen registers; a transposed
// operand comes from two transposing LDS reads).  Used when some clip of the call has T > 16.
namespace {

constexpr int kT2Rows = 32;

template <int D>
struct T2Cfg {
  static constexpr int kTileBytes = kT2Rows * D * 2;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kLoadsPerTile = kT2Rows * kChunksPerRow / 64;
};

template <int D>
__device__ __forceinline__ void gather_tile32(const __bf16* base, const TUnit& u, uint32_t row_bytes,
                                              uint32_t lds_tile, int lane) {
  using Cfg = T2Cfg<D>;
#pragma unroll
  for (int x = 0; x < Cfg::kLoadsPerTile; ++x) {
    const int p = x * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    const int chunk = (p % Cfg::kChunksPerRow) ^ swz<D>(r);
    const uint32_t off = (uint32_t)(u.first_row + min(r, u.T - 1) * u.hw) * row_bytes +
                         (uint32_t)(u.head * D * 2 + chunk * 16);
    lds_dma16(base, off, lds_tile + x * 1024);
  }
}

// Row operands: lane l holds row l%32, columns ks*16 + 8*(l/32)..+7.
template <int D>
__device__ __forceinline__ void read_rows32(const char* tile, int lane, bf16x8 (&f)[D / 16]) {
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) f[ks] = lds_read_b128(tile, tile_off<D>(lane & 31, ks * 16 + 8 * (lane >> 5)));
}

// Transposed operand X^T[d = db*32 + ..][rows 16*s2 ..] of a tile, for the contraction over rows.
template <int D>
__device__ __forceinline__ bf16x8 read_tr32(const char* tile, int lane, int db, int s2) {
  const int g = lane >> 5;
  const int col = db * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const int row = 16 * s2 + 4 * g + ((lane & 15) >> 2);
  return join_tr(lds_read_tr(tile, tile_off<D>(row, col)), lds_read_tr(tile, tile_off<D>(row + 8, col)));
}

// Store an accumulator tile C[d = db*32 + 8*(r/4) + 4*(l/32) + r%4][token = l%32] as bf16 of row `token`.
template <int D>
__device__ __forceinline__ void store_tile32(__bf16* base, const TUnit& u, size_t row_stride, int lane,
                                             int db, const f32x16& c, float mul) {
  if ((lane & 31) < u.T) {
    const size_t row = (size_t)(u.first_row + (lane & 31) * u.hw);
    __bf16* p = base + row * row_stride + (size_t)u.head * D + db * 32 + 4 * (lane >> 5);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      f32x4 o = {c[4 * q4] * mul, c[4 * q4 + 1] * mul, c[4 * q4 + 2] * mul, c[4 * q4 + 3] * mul};
      *reinterpret_cast<bf16x4*>(p + 8 * q4) = to_bf16x4(o);
    }
  }
}

__device__ __forceinline__ bf16x8 half_to_bf16(const f32x16& x, int s2) {
  f32x8 a;
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = x[8 * s2 + e];
  return to_bf16x8(a);
}

}  // namespace

template <int D>
__global__ __launch_bounds__(kTWaves * 64) void tattn32_fwd_kernel(const __bf16* __restrict__ q,
                                                                   const __bf16* __restrict__ k,
                                                                   const __bf16* __restrict__ v,
                                                                   __bf16* __restrict__ out,
                                                                   const TemporalTable tab, int n_heads,
                                                                   float scale_log2) {
  using Cfg = T2Cfg<D>;
  constexpr int TB = Cfg::kTileBytes;
  constexpr int KS = D / 16, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  TUnit u;
  if (!temporal_unit(tab, n_heads, u)) return;   // whole wavefronts leave; there are no barriers
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  char* mine = smem + wave * 3 * TB;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(mine));
  gather_tile32<D>(q, u, row_bytes, lds0, lane);
  gather_tile32<D>(k, u, row_bytes, lds0 + TB, lane);
  gather_tile32<D>(v, u, row_bytes, lds0 + 2 * TB, lane);
  wait_vmcnt<0>();

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 qf[KS], kf[KS];
  read_rows32<D>(mine, lane, qf);
  read_rows32<D>(mine + TB, lane, kf);
  f32x16 st = zero16;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) st = mfma32(kf[ks], qf[ks], st);
  // lane: query l%32; register r: key 8*(r/4) + 4g + r%4
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    if (8 * (r >> 2) + 4 * g + (r & 3) >= u.T) st[r] = -INFINITY;
    mx = fmaxf(mx, st[r]);
  }
  const float m2 = pair_max(mx) * scale_log2;
  f32x16 p;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    p[r] = fast_exp2(st[r] * scale_log2 - m2);
    sum += p[r];
  }
  const float inv = 1.0f / pair_sum(sum);
#pragma unroll
  for (int r = 0; r < 16; ++r) p[r] *= inv;
  const bf16x8 pb0 = half_to_bf16(p, 0), pb1 = half_to_bf16(p, 1);
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    f32x16 o = mfma32(read_tr32<D>(mine + 2 * TB, lane, db, 0), pb0, zero16);
    o = mfma32(read_tr32<D>(mine + 2 * TB, lane, db, 1), pb1, o);
    store_tile32<D>(out, u, row_stride, lane, db, o, 1.0f);
  }
}

template <int D>
__global__ __launch_bounds__(kTWaves * 64) void tattn32_bwd_kernel(const __bf16* __restrict__ q,
                                                                   const __bf16* __restrict__ k,
                                                                   const __bf16* __restrict__ v,
                                                                   const __bf16* __restrict__ dout,
                                                                   __bf16* __restrict__ dq,
                                                                   __bf16* __restrict__ dk,
                                                                   __bf16* __restrict__ dv,
                                                                   const TemporalTable tab, int n_heads,
                                                                   float scale, float scale_log2) {
  using Cfg = T2Cfg<D>;
  constexpr int TB = Cfg::kTileBytes;
  constexpr int KS = D / 16, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  TUnit u;
  if (!temporal_unit(tab, n_heads, u)) return;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  char* qt = smem + wave * 4 * TB;
  char* kt = qt + TB;
  char* vt = qt + 2 * TB;
  char* dot = qt + 3 * TB;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(qt));
  gather_tile32<D>(q, u, row_bytes, lds0, lane);
  gather_tile32<D>(k, u, row_bytes, lds0 + TB, lane);
  gather_tile32<D>(v, u, row_bytes, lds0 + 2 * TB, lane);
  gather_tile32<D>(dout, u, row_bytes, lds0 + 3 * TB, lane);
  wait_vmcnt<0>();

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 qf[KS], kf[KS], vf[KS], df[KS];
  read_rows32<D>(qt, lane, qf);
  read_rows32<D>(kt, lane, kf);
  read_rows32<D>(vt, lane, vf);
  read_rows32<D>(dot, lane, df);
  // "A": lane = query, registers = keys (S^T, dP^T);  "B": lane = key, registers = queries (S, dP)
  f32x16 sA = zero16, dpA = zero16;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    sA = mfma32(kf[ks], qf[ks], sA);
    dpA = mfma32(vf[ks], df[ks], dpA);
  }
  // softmax statistics per query, in orientation A
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    if (8 * (r >> 2) + 4 * g + (r & 3) >= u.T) sA[r] = -INFINITY;
    mx = fmaxf(mx, sA[r]);
  }
  const float m2 = pair_max(mx) * scale_log2;
  f32x16 pA;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    pA[r] = fast_exp2(sA[r] * scale_log2 - m2);
    sum += pA[r];
  }
  sum = pair_sum(sum);
  const float lse2 = m2 + __log2f(sum);      // P = exp2(s*scale_log2 - lse2)
  const float inv = 1.0f / sum;
  float dl = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    pA[r] *= inv;
    dl += pA[r] * dpA[r];
  }
  const float delta = pair_sum(dl);          // Delta_i = sum_j P_ij dP_ij
  f32x16 dsA;
#pragma unroll
  for (int r = 0; r < 16; ++r) dsA[r] = pA[r] * (dpA[r] - delta);
  {
    // dQ^T[d, i] = scale sum_j K[j, d] dS^T[j, i]
    const bf16x8 d0 = half_to_bf16(dsA, 0), d1 = half_to_bf16(dsA, 1);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      f32x16 o = mfma32(read_tr32<D>(kt, lane, db, 0), d0, zero16);
      o = mfma32(read_tr32<D>(kt, lane, db, 1), d1, o);
      store_tile32<D>(dq, u, row_stride, lane, db, o, scale);
    }
  }
  // orientation B: register r belongs to query i = 8*(r/4) + 4g + r%4, whose statistics lane i holds
  f32x16 sB = zero16, dpB = zero16;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    sB = mfma32(qf[ks], kf[ks], sB);
    dpB = mfma32(df[ks], vf[ks], dpB);
  }
  f32x16 pB, dsB;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = 8 * (r >> 2) + 4 * g + (r & 3);
    const float l2 = __shfl(lse2, i);
    const float dd = __shfl(delta, i);
    const float pv = (i < u.T) ? fast_exp2(sB[r] * scale_log2 - l2) : 0.f;   // padded queries add nothing
    pB[r] = pv;
    dsB[r] = pv * (dpB[r] - dd);
  }
  const bf16x8 p0 = half_to_bf16(pB, 0), p1 = half_to_bf16(pB, 1);
  const bf16x8 s0 = half_to_bf16(dsB, 0), s1 = half_to_bf16(dsB, 1);
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    // dV^T[d, j] = sum_i dO[i, d] P[i, j];  dK^T[d, j] = scale sum_i Q[i, d] dS[i, j]
    f32x16 o = mfma32(read_tr32<D>(dot, lane, db, 0), p0, zero16);
    o = mfma32(read_tr32<D>(dot, lane, db, 1), p1, o);
    store_tile32<D>(dv, u, row_stride, lane, db, o, 1.0f);
    o = mfma32(read_tr32<D>(qt, lane, db, 0), s0, zero16);
    o = mfma32(read_tr32<D>(qt, lane, db, 1), s1, o);
    store_tile32<D>(dk, u, row_stride, lane, db, o, scale);
  }
}

// ---------------------------------------------------------------- more than 32 frames
// Section 4.6 speaks of videos of hundreds of frames.  For clips with T > 32 a wavefront owns one
// 32-row block of one (pixel, head) sequence and walks the sequence's other side in blocks of 32
// with the online softmax of the packed kernels (running reference m, running sum l, rescaled
// accumulators), on the 32 x 32 tiles, lane layouts and LDS helpers of the 17..32-frame kernels.
// Blocks of one sequence are consecutive work units, so the wavefronts that re-read a
// sequence's K/V (or Q/dO) rows run together and find them in cache.
// The backward still takes no workspace: a first kernel writes each query's statistics (lse in
// log2 units and Delta_i = sum_j P_ij dP_ij, two floats) into the first 8 bytes of that query's
// dq row, the dK/dV kernel reads them from there, and the dQ kernel reads its own rows'
// statistics before it overwrites those rows with dq.
namespace {

struct LUnit {
  TUnit u;
  int blk;      // 32-row block of the sequence this wavefront owns
  int n_blk;    // blocks of the sequence
};

__device__ __forceinline__ bool long_unit(const TemporalLTable& tab, int n_heads, LUnit& w) {
  const long long unit = (long long)blockIdx.x * kTWaves + (threadIdx.x >> 6);
  if (unit >= (long long)tab.blk_cu[tab.n] * n_heads) return false;
  int lo = 0, hi = tab.n;            // last clip s with blk_cu[s] * n_heads <= unit (skips empty clips)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((long long)tab.blk_cu[mid] * n_heads <= unit) lo = mid; else hi = mid;
  }
  const int hw = tab.hw[lo];
  const int T = (tab.cu[lo + 1] - tab.cu[lo]) / hw;
  const int nb = (T + kT2Rows - 1) / kT2Rows;
  const long long local = unit - (long long)tab.blk_cu[lo] * n_heads;   // ((pixel * heads + head) * nb + block)
  w.blk = (int)(local % nb);
  w.n_blk = nb;
  const long long ph = local / nb;
  w.u.head = (int)(ph % n_heads);
  w.u.hw = hw;
  w.u.T = T;
  w.u.first_row = tab.cu[lo] + (int)(ph / n_heads);
  return true;
}

// Rows 32*blk .. 32*blk + 31 of the sequence (clamped to its last row) into a swizzled [32][D] tile.
template <int D>
__device__ __forceinline__ void gather_block(const __bf16* base, const TUnit& u, int blk, uint32_t row_bytes,
                                             uint32_t lds_tile, int lane) {
  using Cfg = T2Cfg<D>;
#pragma unroll
  for (int x = 0; x < Cfg::kLoadsPerTile; ++x) {
    const int p = x * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    const int chunk = (p % Cfg::kChunksPerRow) ^ swz<D>(r);
    const uint32_t off = (uint32_t)(u.first_row + min(blk * kT2Rows + r, u.T - 1) * u.hw) * row_bytes +
                         (uint32_t)(u.head * D * 2 + chunk * 16);
    lds_dma16(base, off, lds_tile + x * 1024);
  }
}

// Row operands of block blk straight from global memory: lane l holds row 32*blk + l%32 (clamped),
// columns ks*16 + 8*(l/32)..+7.
template <int D>
__device__ __forceinline__ void load_rows_global(const __bf16* base, const TUnit& u, int blk, size_t row_stride,
                                                 int lane, bf16x8 (&f)[D / 16]) {
  const size_t row = (size_t)(u.first_row + min(blk * kT2Rows + (lane & 31), u.T - 1) * u.hw);
  const __bf16* p = base + row * row_stride + (size_t)u.head * D + 8 * (lane >> 5);
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) f[ks] = *reinterpret_cast<const bf16x8*>(p + ks * 16);
}

// Store an accumulator tile as rows 32*blk + l%32 of the sequence.
template <int D>
__device__ __forceinline__ void store_block(__bf16* base, const TUnit& u, int blk, size_t row_stride, int lane,
                                            int db, const f32x16& c, float mul) {
  const int t = blk * kT2Rows + (lane & 31);
  if (t < u.T) {
    __bf16* p = base + (size_t)(u.first_row + t * u.hw) * row_stride + (size_t)u.head * D + db * 32 + 4 * (lane >> 5);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      f32x4 o = {c[4 * q4] * mul, c[4 * q4 + 1] * mul, c[4 * q4 + 2] * mul, c[4 * q4 + 3] * mul};
      *reinterpret_cast<bf16x4*>(p + 8 * q4) = to_bf16x4(o);
    }
  }
}

// The two statistics of query t of the sequence live in the first 8 bytes of its dq row.
template <int D>
__device__ __forceinline__ float* stat_slot(__bf16* dq, const TUnit& u, int t, size_t row_stride) {
  return reinterpret_cast<float*>(dq + (size_t)(u.first_row + t * u.hw) * row_stride + (size_t)u.head * D);
}

constexpr f32x16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

}  // namespace

// STATS = false: out.  STATS = true (first backward kernel): the queries' statistics into dq rows;
// `v` then also feeds dP^T = V dO^T and `dout` must be given.
template <int D, bool STATS>
__global__ __launch_bounds__(kTWaves * 64) void tattnL_fwd_kernel(const __bf16* __restrict__ q,
                                                                  const __bf16* __restrict__ k,
                                                                  const __bf16* __restrict__ v,
                                                                  const __bf16* __restrict__ dout,
                                                                  __bf16* __restrict__ out,   // out, or dq (statistics)
                                                                  const TemporalLTable tab, int n_heads,
                                                                  float scale_log2) {
  using Cfg = T2Cfg<D>;
  constexpr int TB = Cfg::kTileBytes;
  constexpr int KS = D / 16, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  LUnit w;
  if (!long_unit(tab, n_heads, w)) return;   // whole wavefronts leave; there are no barriers
  const TUnit& u = w.u;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  char* kt = smem + wave * 2 * TB;
  char* vt = kt + TB;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(kt));

  bf16x8 qf[KS], df[KS];
  load_rows_global<D>(q, u, w.blk, row_stride, lane, qf);
  if constexpr (STATS) load_rows_global<D>(dout, u, w.blk, row_stride, lane, df);
  float m = -INFINITY, l = 0.f, dnum = 0.f;   // running reference (log2 units), sum, and sum of e^{s-m} dP
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) oacc[db] = kZero16;

  for (int kb = 0; kb < w.n_blk; ++kb) {
    gather_block<D>(k, u, kb, row_bytes, lds0, lane);
    gather_block<D>(v, u, kb, row_bytes, lds0 + TB, lane);
    wait_vmcnt<0>();
    bf16x8 kf[KS];
    read_rows32<D>(kt, lane, kf);
    f32x16 st = kZero16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) st = mfma32(kf[ks], qf[ks], st);
    // lane: query l%32 of the block; register r: key 32*kb + 8*(r/4) + 4g + r%4
    float mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if (kb * kT2Rows + 8 * (r >> 2) + 4 * g + (r & 3) >= u.T) st[r] = -INFINITY;
      mx = fmaxf(mx, st[r]);
    }
    const float m_new = fmaxf(m, pair_max(mx) * scale_log2);   // every block has a valid key, so m_new is finite
    const float alpha = fast_exp2(m - m_new);                  // 0 for the first block (m = -inf)
    f32x16 p;
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      p[r] = fast_exp2(st[r] * scale_log2 - m_new);
      sum += p[r];
    }
    l = l * alpha + sum;       // (per lane: this lane's half of the keys; halves are added at the end)
    m = m_new;
    if constexpr (STATS) {
      bf16x8 vf[KS];
      read_rows32<D>(vt, lane, vf);
      f32x16 dp = kZero16;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) dp = mfma32(vf[ks], df[ks], dp);
      float dsum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) dsum += p[r] * dp[r];      // p is 0 for masked keys
      dnum = dnum * alpha + dsum;
    } else {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
      const bf16x8 pb0 = half_to_bf16(p, 0), pb1 = half_to_bf16(p, 1);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        oacc[db] = mfma32(read_tr32<D>(vt, lane, db, 0), pb0, oacc[db]);
        oacc[db] = mfma32(read_tr32<D>(vt, lane, db, 1), pb1, oacc[db]);
      }
    }
    // the tiles are overwritten by the next block's loads: every read above must have completed
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  const float l_tot = pair_sum(l);
  if constexpr (STATS) {
    const float d_tot = pair_sum(dnum);       // (both halves of the wavefront take part in the exchange)
    const int t = w.blk * kT2Rows + (lane & 31);
    if (t < u.T && g == 0) {
      float* slot = stat_slot<D>(out, u, t, row_stride);
      slot[0] = m + __log2f(l_tot);           // P = exp2(s * scale_log2 - slot[0])
      slot[1] = d_tot / l_tot;                // Delta
    }
  } else {
    const float inv = 1.0f / l_tot;
#pragma unroll
    for (int db = 0; db < DB; ++db) store_block<D>(out, u, w.blk, row_stride, lane, db, oacc[db], inv);
  }
}

// dK, dV of one 32-key block: walks the sequence's query blocks.
template <int D>
__global__ __launch_bounds__(kTWaves * 64) void tattnL_dkdv_kernel(const __bf16* __restrict__ q,
                                                                   const __bf16* __restrict__ k,
                                                                   const __bf16* __restrict__ v,
                                                                   const __bf16* __restrict__ dout,
                                                                   __bf16* __restrict__ dq,   // statistics (read only here)
                                                                   __bf16* __restrict__ dk, __bf16* __restrict__ dv,
                                                                   const TemporalLTable tab, int n_heads,
                                                                   float scale, float scale_log2) {
  using Cfg = T2Cfg<D>;
  constexpr int TB = Cfg::kTileBytes;
  constexpr int KS = D / 16, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  LUnit w;
  if (!long_unit(tab, n_heads, w)) return;
  const TUnit& u = w.u;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  char* qt = smem + wave * 2 * TB;
  char* dot = qt + TB;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(qt));

  bf16x8 kf[KS], vf[KS];     // this block's key and value rows: lane = key
  load_rows_global<D>(k, u, w.blk, row_stride, lane, kf);
  load_rows_global<D>(v, u, w.blk, row_stride, lane, vf);
  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) { dkacc[db] = kZero16; dvacc[db] = kZero16; }

  for (int qb = 0; qb < w.n_blk; ++qb) {
    gather_block<D>(q, u, qb, row_bytes, lds0, lane);
    gather_block<D>(dout, u, qb, row_bytes, lds0 + TB, lane);
    // statistics of query 32*qb + l%32 (rows past the end: any finite value, their P is zeroed below)
    const int tq = min(qb * kT2Rows + (lane & 31), u.T - 1);
    const float* slot = stat_slot<D>(dq, u, tq, row_stride);
    const float lse2 = slot[0], delta = slot[1];
    wait_vmcnt<0>();
    bf16x8 qf[KS], df[KS];
    read_rows32<D>(qt, lane, qf);
    read_rows32<D>(dot, lane, df);
    // lane = key of this block, register r = query 32*qb + 8*(r/4) + 4g + r%4
    f32x16 sB = kZero16, dpB = kZero16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      sB = mfma32(qf[ks], kf[ks], sB);
      dpB = mfma32(df[ks], vf[ks], dpB);
    }
    f32x16 pB, dsB;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = 8 * (r >> 2) + 4 * g + (r & 3);
      const float l2 = __shfl(lse2, i);
      const float dd = __shfl(delta, i);
      const float pv = (qb * kT2Rows + i < u.T) ? fast_exp2(sB[r] * scale_log2 - l2) : 0.f;   // padded queries add nothing
      pB[r] = pv;
      dsB[r] = pv * (dpB[r] - dd);
    }
    const bf16x8 p0 = half_to_bf16(pB, 0), p1 = half_to_bf16(pB, 1);
    const bf16x8 s0 = half_to_bf16(dsB, 0), s1 = half_to_bf16(dsB, 1);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      // dV^T[d, j] += sum_i dO[i, d] P[i, j];  dK^T[d, j] += sum_i Q[i, d] dS[i, j]
      dvacc[db] = mfma32(read_tr32<D>(dot, lane, db, 0), p0, dvacc[db]);
      dvacc[db] = mfma32(read_tr32<D>(dot, lane, db, 1), p1, dvacc[db]);
      dkacc[db] = mfma32(read_tr32<D>(qt, lane, db, 0), s0, dkacc[db]);
      dkacc[db] = mfma32(read_tr32<D>(qt, lane, db, 1), s1, dkacc[db]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  // keys past the end of the sequence (last block) are never stored
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    store_block<D>(dk, u, w.blk, row_stride, lane, db, dkacc[db], scale);
    store_block<D>(dv, u, w.blk, row_stride, lane, db, dvacc[db], 1.0f);
  }
}

// dQ of one 32-query block: reads the block's statistics from its dq rows, walks the key blocks,
// then overwrites the rows.
template <int D>
__global__ __launch_bounds__(kTWaves * 64) void tattnL_dq_kernel(const __bf16* __restrict__ q,
                                                                 const __bf16* __restrict__ k,
                                                                 const __bf16* __restrict__ v,
                                                                 const __bf16* __restrict__ dout,
                                                                 __bf16* __restrict__ dq,
                                                                 const TemporalLTable tab, int n_heads,
                                                                 float scale, float scale_log2) {
  using Cfg = T2Cfg<D>;
  constexpr int TB = Cfg::kTileBytes;
  constexpr int KS = D / 16, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  LUnit w;
  if (!long_unit(tab, n_heads, w)) return;
  const TUnit& u = w.u;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  char* kt = smem + wave * 2 * TB;
  char* vt = kt + TB;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(kt));

  bf16x8 qf[KS], df[KS];     // lane = query
  load_rows_global<D>(q, u, w.blk, row_stride, lane, qf);
  load_rows_global<D>(dout, u, w.blk, row_stride, lane, df);
  const float* slot = stat_slot<D>(dq, u, min(w.blk * kT2Rows + (lane & 31), u.T - 1), row_stride);
  const float lse2 = slot[0], delta = slot[1];
  f32x16 dqacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) dqacc[db] = kZero16;

  for (int kb = 0; kb < w.n_blk; ++kb) {
    gather_block<D>(k, u, kb, row_bytes, lds0, lane);
    gather_block<D>(v, u, kb, row_bytes, lds0 + TB, lane);
    wait_vmcnt<0>();
    bf16x8 kf[KS], vf[KS];
    read_rows32<D>(kt, lane, kf);
    read_rows32<D>(vt, lane, vf);
    f32x16 sA = kZero16, dpA = kZero16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      sA = mfma32(kf[ks], qf[ks], sA);
      dpA = mfma32(vf[ks], df[ks], dpA);
    }
    f32x16 dsA;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const bool live = kb * kT2Rows + 8 * (r >> 2) + 4 * g + (r & 3) < u.T;
      const float pv = live ? fast_exp2(sA[r] * scale_log2 - lse2) : 0.f;
      dsA[r] = pv * (dpA[r] - delta);
    }
    const bf16x8 d0 = half_to_bf16(dsA, 0), d1 = half_to_bf16(dsA, 1);
#pragma unroll
    for (int db = 0; db < DB; ++db) {   // dQ^T[d, i] += sum_j K[j, d] dS^T[j, i]
      dqacc[db] = mfma32(read_tr32<D>(kt, lane, db, 0), d0, dqacc[db]);
      dqacc[db] = mfma32(read_tr32<D>(kt, lane, db, 1), d1, dqacc[db]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
#pragma unroll
  for (int db = 0; db < DB; ++db) store_block<D>(dq, u, w.blk, row_stride, lane, db, dqacc[db], scale);
}

// Some clip of the run has more than 32 frames: the block-walking kernels serve the whole run.
template <int D>
static hipError_t launch_long(const void* q, const void* k, const void* v, const void* dout,
                              const TemporalTable& tab, int n_heads, float scale, void* o0, void* o1,
                              void* o2, hipStream_t stream) {
  TemporalLTable lt;
  lt.n = tab.n;
  int blocks = 0;
  for (int s = 0; s <= VFM_MAX_SEQS; ++s) {
    lt.cu[s] = tab.cu[s];
    lt.blk_cu[s] = blocks;
    if (s < VFM_MAX_SEQS) {
      lt.hw[s] = tab.hw[s];
      if (s < tab.n && tab.cu[s + 1] > tab.cu[s]) {
        const int T = (tab.cu[s + 1] - tab.cu[s]) / tab.hw[s];
        blocks += tab.hw[s] * ((T + kT2Rows - 1) / kT2Rows);
      }
    }
  }
  const long long n_units = (long long)blocks * n_heads;
  if (n_units == 0) return hipSuccess;
  const dim3 grid((unsigned)((n_units + kTWaves - 1) / kTWaves)), block(kTWaves * 64);
  constexpr int lds = kTWaves * 2 * T2Cfg<D>::kTileBytes;
  const __bf16 *qb = (const __bf16*)q, *kb = (const __bf16*)k, *vb = (const __bf16*)v, *dob = (const __bf16*)dout;
  const float scale_log2 = scale * kLog2eT;
  hipError_t e;
  if (!dout) {
    auto kern = tattnL_fwd_kernel<D, false>;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return launch(kern, grid, block, lds, stream, qb, kb, vb, dob, (__bf16*)o0, lt, n_heads, scale_log2);
  }
  auto stats = tattnL_fwd_kernel<D, true>;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(stats), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  e = launch(stats, grid, block, lds, stream, qb, kb, vb, dob, (__bf16*)o0, lt, n_heads, scale_log2);   // o0 = dq
  if (e != hipSuccess) return e;
  auto dkdv = tattnL_dkdv_kernel<D>;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(dkdv), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  e = launch(dkdv, grid, block, lds, stream, qb, kb, vb, dob, (__bf16*)o0, (__bf16*)o1, (__bf16*)o2, lt, n_heads, scale,
             scale_log2);
  if (e != hipSuccess) return e;
  auto dqk = tattnL_dq_kernel<D>;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(dqk), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  return launch(dqk, grid, block, lds, stream, qb, kb, vb, dob, (__bf16*)o0, lt, n_heads, scale, scale_log2);
}

template <int D>
static hipError_t launch_t(const void* q, const void* k, const void* v, const void* dout,
                           const TemporalTable& tab, int n_heads, float scale, void* o0, void* o1,
                           void* o2, hipStream_t stream) {
  const long long n_units = (long long)tab.pix_cu[tab.n] * n_heads;
  if (n_units == 0) return hipSuccess;
  int max_t = 0;
  for (int s = 0; s < tab.n; ++s)
    if (tab.hw[s] > 0) max_t = std::max(max_t, (tab.cu[s + 1] - tab.cu[s]) / tab.hw[s]);
  if (max_t > kT2Rows) return launch_long<D>(q, k, v, dout, tab, n_heads, scale, o0, o1, o2, stream);
  const bool big = max_t > kTRows;     // some clip has more than 16 frames: 32-row tiles for the call
  const int grid = (int)((n_units + kTWaves - 1) / kTWaves);
  const int tiles = dout ? 4 : 3;
  const int lds = kTWaves * tiles * (big ? T2Cfg<D>::kTileBytes : TCfg<D>::kTileBytes);
  if (!dout) {
    auto kern = big ? tattn32_fwd_kernel<D> : tattn_fwd_kernel<D>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return launch(kern, dim3(grid), dim3(kTWaves * 64), lds, stream, (const __bf16*)q, (const __bf16*)k,
                  (const __bf16*)v, (__bf16*)o0, tab, n_heads, scale * kLog2eT);
  } else {
    auto kern = big ? tattn32_bwd_kernel<D> : tattn_bwd_kernel<D>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return launch(kern, dim3(grid), dim3(kTWaves * 64), lds, stream, (const __bf16*)q, (const __bf16*)k,
                  (const __bf16*)v, (const __bf16*)dout, (__bf16*)o0, (__bf16*)o1, (__bf16*)o2, tab, n_heads,
                  scale, scale * kLog2eT);
  }
}

hipError_t launch_tattn_fwd(const void* q, const void* k, const void* v, const TemporalTable& tab,
                            int n_heads, int head_dim, float scale, void* out, hipStream_t stream) {
  if (head_dim == 128) return launch_t<128>(q, k, v, nullptr, tab, n_heads, scale, out, nullptr, nullptr, stream);
  return launch_t<64>(q, k, v, nullptr, tab, n_heads, scale, out, nullptr, nullptr, stream);
}

hipError_t launch_tattn_bwd(const void* q, const void* k, const void* v, const void* dout,
                            const TemporalTable& tab, int n_heads, int head_dim, float scale, void* dq,
                            void* dk, void* dv, hipStream_t stream) {
  if (head_dim == 128) return launch_t<128>(q, k, v, dout, tab, n_heads, scale, dq, dk, dv, stream);
  return launch_t<64>(q, k, v, dout, tab, n_heads, scale, dq, dk, dv, stream);
}

}  // namespace vfm
