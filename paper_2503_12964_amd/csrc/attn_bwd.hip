// Packed variable-length attention backward for gfx950 (bf16 MFMA, fp32 accumulate).
//
// Three kernels, no atomics (device-wide fp32 atomics are executed at the memory side on
// this chip and were measured to bound the fused variant), so every output is written
// once and the result is bitwise reproducible:
//   bwd_prepare : Delta[h,i] = sum_d dO[i,h,d] O[i,h,d]
//   bwd_dkdv    : one workgroup owns kBC key/value rows of one (clip, head); its four
//                 wavefronts own 32 of those rows each and keep their K and V rows, and
//                 their dK^T / dV^T accumulators, in registers.  The workgroup walks the
//                 clip's query rows in tiles of kBQ, staged (Q, dO, lse, Delta) through
//                 LDS, and per tile computes
//                     S  = Q K^T,  dP = dO V^T            (A = Q/dO rows, B = K/V registers)
//                     P  = exp(scale*S - lse),  dS = P o (dP - Delta)
//                     dV^T += dO^T P,  dK^T += Q^T dS     (A = transposing LDS reads, B = P/dS registers)
//   bwd_dq      : one workgroup owns a query tile (like the forward kernel) and streams
//                 the clip's K/V tiles through LDS:
//                     S^T = K Q^T,  dP^T = V dO^T          (A = K/V rows, B = Q/dO registers)
//                     dS^T = P^T o (dP^T - Delta)          (lse, Delta are per-lane scalars)
//                     dQ^T += K^T dS^T                     (A = transposing reads of the K tile)
//                 S and dP are recomputed here (7 GEMMs in total instead of 5).
#include "vfm_common.h"

namespace vfm {

constexpr int kBwdWaves = 4;
constexpr int kBwdBC = 128;  // key/value rows per workgroup (32 per wavefront)
constexpr int kBwdBQ = 64;   // query rows per inner step
constexpr float kLog2eB = 1.4426950408889634f;

// ---------------------------------------------------------------- prepare
template <int D>
__global__ __launch_bounds__(256) void bwd_prepare_kernel(const u32x4* __restrict__ out,
                                                          const u32x4* __restrict__ dout,
                                                          float* __restrict__ delta, int total,
                                                          int n_heads) {
  constexpr int kLanesPerRow = D / 8;
  constexpr int kTokPerBlock = 256 / kLanesPerRow;
  const int tok = blockIdx.x * kTokPerBlock + threadIdx.x / kLanesPerRow;
  const int chunk = threadIdx.x % kLanesPerRow;
  const bool valid = tok < total;
  const int tk = valid ? tok : total - 1;
  for (int h = 0; h < n_heads; ++h) {
    const size_t row = (size_t)tk * n_heads + h;
    const u32x4 a = out[row * kLanesPerRow + chunk];
    const u32x4 b = dout[row * kLanesPerRow + chunk];
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s += __builtin_bit_cast(float, a[e] << 16) * __builtin_bit_cast(float, b[e] << 16);
      s += __builtin_bit_cast(float, a[e] & 0xffff0000u) * __builtin_bit_cast(float, b[e] & 0xffff0000u);
    }
#pragma unroll
    for (int o = kLanesPerRow / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, kLanesPerRow);
    if (valid && chunk == 0) delta[(size_t)h * total + tok] = s;
  }
}

// ---------------------------------------------------------------- dK, dV
template <int D>
struct BwdCfg {
  static constexpr int kTileBytes = kBwdBQ * D * 2;               // one Q or dO tile
  static constexpr int kStageBytes = 2 * kTileBytes + 2 * kBwdBQ * 4;  // Q, dO, lse, Delta
  static constexpr int kLdsBytes = 2 * kStageBytes;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kChunksPerThread = kBwdBQ * kChunksPerRow / (kBwdWaves * 64);
};

template <int D>
__global__ __launch_bounds__(kBwdWaves * 64, 1)
void attn_bwd_dkdv_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                     const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                     const float* __restrict__ lse, const float* __restrict__ delta,
                     __bf16* __restrict__ dk, __bf16* __restrict__ dv,
                     const SegTable segs, const UnitMap um,
                     int total, int n_heads, float scale, float scale_log2) {
  using Cfg = BwdCfg<D>;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int NIB = kBwdBQ / 32;              // query blocks per step (2)
  constexpr int CPT = Cfg::kChunksPerThread;

  extern __shared__ __attribute__((aligned(16))) char smem[];

  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  int seg_a, seg_b, j0;
  find_tile(segs, kBwdBC, tile, seg_a, seg_b, j0);

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int c = lane & 31;
  const int g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const size_t head_off = (size_t)head * D;

  // ---- this wavefront's key/value rows as B operands (lane: row c, columns ks*16+8g..)
  const int jrow = j0 + wave * 32 + c;
  const bool jvalid = jrow < seg_b;
  const bool tail_kv = (j0 + kBwdBC > seg_b);
  bf16x8 kreg[KS], vreg[KS];
  {
    const size_t off = (size_t)min(jrow, seg_b - 1) * row_stride + head_off + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kreg[ks] = *reinterpret_cast<const bf16x8*>(k + off + ks * 16);
      vreg[ks] = *reinterpret_cast<const bf16x8*>(v + off + ks * 16);
    }
  }
  // ---- staging of Q / dO / lse / Delta tiles
  int st_row[CPT], st_chunk[CPT], st_lds[CPT];
#pragma unroll
  for (int x = 0; x < CPT; ++x) {
    const int idx = tid + x * (kBwdWaves * 64);
    st_row[x] = idx / Cfg::kChunksPerRow;
    st_chunk[x] = idx % Cfg::kChunksPerRow;
    st_lds[x] = tile_off<D>(st_row[x], st_chunk[x] * 8);
  }
  u32x4 qst[CPT], dost[CPT];
  float stat = 0.f;  // threads 0..63: lse (log2 units), 64..127: Delta
  const float* lse_h = lse + (size_t)head * total;
  const float* delta_h = delta + (size_t)head * total;
  auto load_tile = [&](int q0) {
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      const int r = min(q0 + st_row[x], seg_b - 1);
      const size_t off = (size_t)r * row_stride + head_off + st_chunk[x] * 8;
      qst[x] = *reinterpret_cast<const u32x4*>(q + off);
      dost[x] = *reinterpret_cast<const u32x4*>(dout + off);
    }
    if (tid < 2 * kBwdBQ) {
      const int r = q0 + (tid & (kBwdBQ - 1));
      if (tid < kBwdBQ) stat = (r < seg_b) ? lse_h[r] * kLog2eB : INFINITY;  // +inf => P = 0
      else stat = (r < seg_b) ? delta_h[r] : 0.f;
    }
  };
  auto store_tile = [&](int stage) {
    char* qt = smem + stage * Cfg::kStageBytes;
    char* dot = qt + Cfg::kTileBytes;
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      *reinterpret_cast<u32x4*>(qt + st_lds[x]) = qst[x];
      *reinterpret_cast<u32x4*>(dot + st_lds[x]) = dost[x];
    }
    if (tid < 2 * kBwdBQ) reinterpret_cast<float*>(qt + 2 * Cfg::kTileBytes)[tid] = stat;
  };

  // ---- per-lane LDS offsets.  The swizzles XOR low byte-offset bits with a function
  // of the low row bits only, so one base per lane serves every k-step / block:
  //   Q/dO rows as A operand (row ib*32 + c, columns ks*16 + 8g):
  //       off = (rbase ^ (ks << 5)) + ib*32*rowbytes
  //   Q^T/dO^T as A operand through transposing reads (same slot binding as the
  //   forward kernel's V^T operand):
  //       off = (tbase[t] ^ (db << 6)) + (ib*32 + 16*s2)*rowbytes
  constexpr int RB = D * 2;
  const int rbase = tile_off<D>(c, 8 * g);
  int tbase[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    tbase[t] = tile_off<D>(8 * t + 4 * g + ((lane & 15) >> 2),
                           16 * ((lane >> 4) & 1) + 4 * (lane & 3));
  }

  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkacc[db][r] = 0.f; dvacc[db][r] = 0.f; }

  const int n_q = seg_b - seg_a;
  const int n_steps = (n_q + kBwdBQ - 1) / kBwdBQ;

  load_tile(seg_a);
  store_tile(0);
  __syncthreads();

  for (int t = 0; t < n_steps; ++t) {
    const int q0 = seg_a + t * kBwdBQ;
    const bool more = (t + 1 < n_steps);
    if (more) load_tile(q0 + kBwdBQ);

    const char* qt = smem + (t & 1) * Cfg::kStageBytes;
    const char* dot = qt + Cfg::kTileBytes;
    const float* lse_s = reinterpret_cast<const float*>(qt + 2 * Cfg::kTileBytes);
    const float* delta_s = lse_s + kBwdBQ;

#pragma unroll
    for (int ib = 0; ib < NIB; ++ib) {
      f32x16 sacc, dpacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; dpacc[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sacc = mfma32(lds_read_b128(qt, (rbase ^ (ks << 5)) + ib * 32 * RB), kreg[ks], sacc);
        dpacc = mfma32(lds_read_b128(dot, (rbase ^ (ks << 5)) + ib * 32 * RB), vreg[ks], dpacc);
      }
      // P and dS for rows i = ib*32 + 8*q4 + 4g + e, column j = this lane's key
      f32x16 p, ds;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + ib * 32 + 8 * q4 + 4 * g);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(delta_s + ib * 32 + 8 * q4 + 4 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = q4 * 4 + e;
          float pv = fast_exp2(sacc[r] * scale_log2 - l4[e]);
          if (tail_kv) pv = jvalid ? pv : 0.f;
          p[r] = pv;
          ds[r] = pv * (dpacc[r] - d4[e]);
        }
      }
      bf16x8 pb[2], dsb8[2];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        f32x8 a, b;
#pragma unroll
        for (int e = 0; e < 8; ++e) { a[e] = p[8 * s2 + e]; b[e] = ds[8 * s2 + e]; }
        pb[s2] = to_bf16x8(a);
        dsb8[s2] = to_bf16x8(b);
      }
      // dV^T += dO^T P ; dK^T += Q^T dS
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int o0 = (tbase[0] ^ (db << 6)) + (ib * 32 + 16 * s2) * RB;
          const int o1 = (tbase[1] ^ (db << 6)) + (ib * 32 + 16 * s2) * RB;
          const bf16x8 doa = join_tr(lds_read_tr(dot, o0), lds_read_tr(dot, o1));
          dvacc[db] = mfma32(doa, pb[s2], dvacc[db]);
          const bf16x8 qa = join_tr(lds_read_tr(qt, o0), lds_read_tr(qt, o1));
          dkacc[db] = mfma32(qa, dsb8[s2], dkacc[db]);
        }
    }

    if (more) store_tile((t + 1) & 1);
    __syncthreads();

  }

  // ---- epilogue: dK (scaled) and dV for this lane's key row
  if (jvalid) {
    __bf16* dkp = dk + (size_t)jrow * row_stride + head_off + 4 * g;
    __bf16* dvp = dv + (size_t)jrow * row_stride + head_off + 4 * g;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[e] = dkacc[db][q4 * 4 + e] * scale;
          b[e] = dvacc[db][q4 * 4 + e];
        }
        *reinterpret_cast<bf16x4*>(dkp + db * 32 + q4 * 8) = to_bf16x4(a);
        *reinterpret_cast<bf16x4*>(dvp + db * 32 + q4 * 8) = to_bf16x4(b);
      }
  }
}

// ---------------------------------------------------------------- dQ
constexpr int kDqWaves = 4;
constexpr int kDqBC = 64;   // key/value rows per LDS tile

template <int D, int NI>
struct DqCfg {
  static constexpr int kBR = kDqWaves * NI * 32;        // query rows per workgroup
  static constexpr int kTileBytes = kDqBC * D * 2;      // one K or V tile
  static constexpr int kLdsBytes = 4 * kTileBytes;      // K, V x 2 stages
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kChunksPerThread = kDqBC * kChunksPerRow / (kDqWaves * 64);
};

template <int D, int NI>
__global__ __launch_bounds__(kDqWaves * 64, 1)
void attn_bwd_dq_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                        const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                        const float* __restrict__ lse, const float* __restrict__ delta,
                        __bf16* __restrict__ dq, const SegTable segs, const UnitMap um,
                        int total, int n_heads, float scale, float scale_log2) {
  using Cfg = DqCfg<D, NI>;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int JB = kDqBC / 32;
  constexpr int CPT = Cfg::kChunksPerThread;
  constexpr int RB = D * 2;

  extern __shared__ __attribute__((aligned(16))) char smem[];

  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  int seg_a, seg_b, q0;
  find_tile(segs, Cfg::kBR, tile, seg_a, seg_b, q0);

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int c = lane & 31;
  const int g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const size_t head_off = (size_t)head * D;
  const __bf16* kbase = k + head_off;
  const __bf16* vbase = v + head_off;

  // ---- Q and dO rows as B operands; lse (log2 units) and Delta are per-lane scalars
  bf16x8 qreg[NI][KS], doreg[NI][KS];
  float lse2[NI], dlt[NI];
  int qrow[NI];
#pragma unroll
  for (int ib = 0; ib < NI; ++ib) {
    qrow[ib] = q0 + (wave * NI + ib) * 32 + c;
    const int r = min(qrow[ib], seg_b - 1);
    const size_t off = (size_t)r * row_stride + head_off + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qreg[ib][ks] = *reinterpret_cast<const bf16x8*>(q + off + ks * 16);
      doreg[ib][ks] = *reinterpret_cast<const bf16x8*>(dout + off + ks * 16);
    }
    lse2[ib] = lse[(size_t)head * total + r] * kLog2eB;
    dlt[ib] = delta[(size_t)head * total + r];
  }

  // ---- K/V staging (same scheme as the forward kernel)
  int st_row[CPT], st_chunk[CPT], st_lds[CPT];
#pragma unroll
  for (int x = 0; x < CPT; ++x) {
    const int idx = tid + x * (kDqWaves * 64);
    st_row[x] = idx / Cfg::kChunksPerRow;
    st_chunk[x] = idx % Cfg::kChunksPerRow;
    st_lds[x] = tile_off<D>(st_row[x], st_chunk[x] * 8);
  }
  u32x4 kst[CPT], vst[CPT];
  auto load_tile = [&](int j0) {
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      const int r = min(j0 + st_row[x], seg_b - 1);
      const size_t off = (size_t)r * row_stride + st_chunk[x] * 8;
      kst[x] = *reinterpret_cast<const u32x4*>(kbase + off);
      vst[x] = *reinterpret_cast<const u32x4*>(vbase + off);
    }
  };
  auto store_tile = [&](int stage) {
    char* kt = smem + stage * 2 * Cfg::kTileBytes;
    char* vt = kt + Cfg::kTileBytes;
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      *reinterpret_cast<u32x4*>(kt + st_lds[x]) = kst[x];
      *reinterpret_cast<u32x4*>(vt + st_lds[x]) = vst[x];
    }
  };

  // K/V rows as A operand: off = (rbase ^ (ks << 5)) + jb*32*RB
  // K^T as A operand (transposing reads): off = (tbase[t] ^ (db << 6)) + (jb*32 + 16*s2)*RB
  const int rbase = tile_off<D>(c, 8 * g);
  int tbase[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    tbase[t] = tile_off<D>(8 * t + 4 * g + ((lane & 15) >> 2),
                           16 * ((lane >> 4) & 1) + 4 * (lane & 3));

  f32x16 dqacc[NI][DB];
#pragma unroll
  for (int ib = 0; ib < NI; ++ib)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dqacc[ib][db][r] = 0.f;

  const int n_tiles = (seg_b - seg_a + kDqBC - 1) / kDqBC;
  load_tile(seg_a);
  store_tile(0);
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = seg_a + t * kDqBC;
    const bool more = (t + 1 < n_tiles);
    if (more) load_tile(j0 + kDqBC);
    const char* kt = smem + (t & 1) * 2 * Cfg::kTileBytes;
    const char* vt = kt + Cfg::kTileBytes;
    const bool tail = (j0 + kDqBC > seg_b);

#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
      f32x16 sacc[NI], dpacc[NI];
#pragma unroll
      for (int ib = 0; ib < NI; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[ib][r] = 0.f; dpacc[ib][r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = (rbase ^ (ks << 5)) + jb * 32 * RB;
        const bf16x8 ka = lds_read_b128(kt, off);
        const bf16x8 va = lds_read_b128(vt, off);
#pragma unroll
        for (int ib = 0; ib < NI; ++ib) {
          sacc[ib] = mfma32(ka, qreg[ib][ks], sacc[ib]);
          dpacc[ib] = mfma32(va, doreg[ib][ks], dpacc[ib]);
        }
      }
      bf16x8 dsb[NI][2];
#pragma unroll
      for (int ib = 0; ib < NI; ++ib) {
        f32x16 ds;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float pv = fast_exp2(sacc[ib][r] * scale_log2 - lse2[ib]);
          if (tail) {
            const int j = j0 + jb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            pv = (j < seg_b) ? pv : 0.f;
          }
          ds[r] = pv * (dpacc[ib][r] - dlt[ib]);
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          f32x8 a;
#pragma unroll
          for (int e = 0; e < 8; ++e) a[e] = ds[8 * s2 + e];
          dsb[ib][s2] = to_bf16x8(a);
        }
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int o0 = (tbase[0] ^ (db << 6)) + (jb * 32 + 16 * s2) * RB;
          const int o1 = (tbase[1] ^ (db << 6)) + (jb * 32 + 16 * s2) * RB;
          const bf16x8 kta = join_tr(lds_read_tr(kt, o0), lds_read_tr(kt, o1));
#pragma unroll
          for (int ib = 0; ib < NI; ++ib) dqacc[ib][db] = mfma32(kta, dsb[ib][s2], dqacc[ib][db]);
        }
    }

    if (more) store_tile((t + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: dq = bf16(scale * dQ^T)
#pragma unroll
  for (int ib = 0; ib < NI; ++ib) {
    const int i = qrow[ib];
    if (i < seg_b) {
      __bf16* op = dq + (size_t)i * row_stride + head_off + 4 * g;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = dqacc[ib][db][q4 * 4 + e] * scale;
          *reinterpret_cast<bf16x4*>(op + db * 32 + q4 * 8) = to_bf16x4(o);
        }
    }
  }
}

template <int D>
static hipError_t launch_bwd_d(const void* q, const void* k, const void* v, const void* out,
                               const float* lse, const void* dout, const SegTable& segs, int total,
                               int n_heads, float scale, void* dq, void* dk, void* dv,
                               float* delta, hipStream_t stream) {
  if (total == 0) return hipSuccess;
  {
    constexpr int kTokPerBlock = 256 / (D / 8);
    const int grid = (total + kTokPerBlock - 1) / kTokPerBlock;
    bwd_prepare_kernel<D><<<grid, 256, 0, stream>>>((const u32x4*)out, (const u32x4*)dout, delta,
                                                    total, n_heads);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    using Cfg = BwdCfg<D>;
    int tiles = 0;
    for (int s = 0; s < segs.n; ++s) tiles += (segs.len[s] + kBwdBC - 1) / kBwdBC;
    if (tiles == 0) return hipSuccess;
    UnitMap um;
    um.tiles_per_head = tiles;
    um.n_units = tiles * n_heads;
    um.chunk = (um.n_units + kNumXcd - 1) / kNumXcd;
    auto kern = attn_bwd_dkdv_kernel<D>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    kern<<<um.chunk * kNumXcd, kBwdWaves * 64, Cfg::kLdsBytes, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)dout, lse, delta,
        (__bf16*)dk, (__bf16*)dv, segs, um, total, n_heads, scale, scale * kLog2eB);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    constexpr int NI = 2;
    using Cfg = DqCfg<D, NI>;
    int tiles = 0;
    for (int s = 0; s < segs.n; ++s) tiles += (segs.len[s] + Cfg::kBR - 1) / Cfg::kBR;
    UnitMap um;
    um.tiles_per_head = tiles;
    um.n_units = tiles * n_heads;
    um.chunk = (um.n_units + kNumXcd - 1) / kNumXcd;
    auto kern = attn_bwd_dq_kernel<D, NI>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    kern<<<um.chunk * kNumXcd, kDqWaves * 64, Cfg::kLdsBytes, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)dout, lse, delta,
        (__bf16*)dq, segs, um, total, n_heads, scale, scale * kLog2eB);
    return hipGetLastError();
  }
}

hipError_t launch_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                           const float* lse, const void* dout, const SegTable& segs, int total,
                           int n_heads, int head_dim, float scale, void* dq, void* dk, void* dv,
                           float* delta, hipStream_t stream) {
  if (head_dim == 128)
    return launch_bwd_d<128>(q, k, v, out, lse, dout, segs, total, n_heads, scale, dq, dk, dv, delta, stream);
  return launch_bwd_d<64>(q, k, v, out, lse, dout, segs, total, n_heads, scale, dq, dk, dv, delta, stream);
}

}  // namespace vfm
