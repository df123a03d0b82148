// Packed variable-length attention backward for gfx950 (bf16 MFMA, fp32 accumulate).
//
// Three kernels:
//   bwd_prepare : Delta[h,i] = sum_d dO[i,h,d] O[i,h,d]  and zero the fp32 dq accumulator
//   bwd_main    : one workgroup owns kBC key/value rows of one (clip, head); its four
//                 wavefronts own 32 of those rows each and keep their K and V rows, and
//                 their dK^T / dV^T accumulators, in registers.  The workgroup walks the
//                 clip's query rows in tiles of kBQ, staged (Q, dO, lse, Delta) through
//                 LDS, and per tile computes
//                     S  = Q K^T,  dP = dO V^T            (A = Q/dO rows, B = K/V registers)
//                     P  = exp(scale*S - lse),  dS = P o (dP - Delta)
//                     dV^T += dO^T P,  dK^T += Q^T dS     (A = transposing LDS reads, B = P/dS registers)
//                 then exchanges dS through LDS so that each wavefront can form a
//                 32-column slice of  dQ = dS K  over all kBC keys and add it to the fp32
//                 accumulator with atomics.
//   bwd_finish  : dq = bf16(scale * accumulator)
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
                                                          float* __restrict__ delta,
                                                          f32x4* __restrict__ dq_acc, int total,
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
    if (valid) {
      if (chunk == 0) delta[(size_t)h * total + tok] = s;
      const f32x4 z = {0.f, 0.f, 0.f, 0.f};
      dq_acc[(row * kLanesPerRow + chunk) * 2] = z;
      dq_acc[(row * kLanesPerRow + chunk) * 2 + 1] = z;
    }
  }
}

// ---------------------------------------------------------------- finish
__global__ __launch_bounds__(256) void bwd_finish_kernel(const f32x8* __restrict__ dq_acc,
                                                         bf16x8* __restrict__ dq, size_t n8,
                                                         float scale) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  f32x8 a = __builtin_nontemporal_load(dq_acc + i);
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] *= scale;
  dq[i] = to_bf16x8(a);
}

// ---------------------------------------------------------------- main
template <int D>
struct BwdCfg {
  static constexpr int kTileBytes = kBwdBQ * D * 2;               // one Q or dO tile
  static constexpr int kStageBytes = 2 * kTileBytes + 2 * kBwdBQ * 4;  // Q, dO, lse, Delta
  static constexpr int kDsBytes = kBwdBC * kBwdBQ * 2;            // one dS buffer
  static constexpr int kLdsBytes = 2 * kStageBytes + 2 * kDsBytes;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kChunksPerThread = kBwdBQ * kChunksPerRow / (kBwdWaves * 64);
};

// dS exchange buffer: [kBwdBC key rows][kBwdBQ query columns] bf16, addressed in
// 8-byte quads (4 query columns).  The quad index is XOR-ed with a permutation of
// key-row bits 1..4 so that the per-lane 8-byte writes (32 consecutive key rows,
// one quad) and the transposing reads (4 consecutive key rows x 64 bytes) both
// spread over all banks.
__device__ __forceinline__ int ds_off(int j, int quad) {
  const int f = (((j >> 1) & 1) << 3) | ((j >> 2) & 1) | (((j >> 3) & 1) << 1) | (((j >> 4) & 1) << 2);
  return j * (kBwdBQ * 2) + ((quad ^ f) << 3);
}

template <int D>
__global__ __launch_bounds__(kBwdWaves * 64, 1)
void attn_bwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                     const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                     const float* __restrict__ lse, const float* __restrict__ delta,
                     __bf16* __restrict__ dk, __bf16* __restrict__ dv,
                     float* __restrict__ dq_acc, const SegTable segs, const UnitMap um,
                     int total, int n_heads, float scale, float scale_log2) {
  using Cfg = BwdCfg<D>;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int NIB = kBwdBQ / 32;              // query blocks per step (2)
  constexpr int CPT = Cfg::kChunksPerThread;
  constexpr int KSJ = kBwdBC / 16;              // k-steps of the dQ contraction over keys
  constexpr int NDQ = (NIB * DB) / kBwdWaves;   // dQ blocks (32x32) per wavefront per step

  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* ds_base = smem + 2 * Cfg::kStageBytes;

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
  // ---- K as B operand of dQ = dS K over all kBC keys: lane holds column d = dq_db*32 + c,
  // contraction slots (g, e) of k-step s are key rows 16s + 8g + e.
  const int dq_db = (NDQ == 2) ? wave : (wave & 1);
  bf16x8 kq[KSJ];
  {
    const __bf16* kp = k + head_off + dq_db * 32 + c;
#pragma unroll
    for (int s = 0; s < KSJ; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int r = min(j0 + 16 * s + 8 * g + e, seg_b - 1);
        kq[s][e] = kp[(size_t)r * row_stride];
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
  //   dS write (key row wave*32 + c, quad ib*8 + q4*2 + g):
  //       off = dswbase ^ ((ib*8 + q4*2) << 3)
  //   dS transposing read for k-step s (key rows 16s + 8g + 4t + ((lane&15)>>2)):
  //       off = (dsrbase[t] ^ ((s & 1) << 5) ^ (ib << 6)) + 16*s*dsrowbytes
  constexpr int RB = D * 2;
  constexpr int DSRB = kBwdBQ * 2;
  const int rbase = tile_off<D>(c, 8 * g);
  int tbase[2], dsrbase[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    tbase[t] = tile_off<D>(8 * t + 4 * g + ((lane & 15) >> 2),
                           16 * ((lane >> 4) & 1) + 4 * (lane & 3));
    dsrbase[t] = ds_off(8 * g + 4 * t + ((lane & 15) >> 2), 4 * ((lane >> 4) & 1) + (lane & 3));
  }
  const int dswbase = ds_off(wave * 32 + c, g);

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
    char* dsb = ds_base + (t & 1) * Cfg::kDsBytes;

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
        // dS -> LDS, two quads (query columns 8*(2*s2+x) + 4g .. +3)
        const u32x4 w = __builtin_bit_cast(u32x4, dsb8[s2]);
        u32x2 w0 = {w[0], w[1]}, w1 = {w[2], w[3]};
        *reinterpret_cast<u32x2*>(dsb + (dswbase ^ ((ib * 8 + (2 * s2) * 2) << 3))) = w0;
        *reinterpret_cast<u32x2*>(dsb + (dswbase ^ ((ib * 8 + (2 * s2 + 1) * 2) << 3))) = w1;
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

    // ---- dQ slice: rows of block ib, columns dq_db*32 + c, contraction over all kBC keys
#pragma unroll
    for (int x = 0; x < NDQ; ++x) {
      const int ib = (NDQ == 2) ? x : (wave >> 1);
      f32x16 dqacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) dqacc[r] = 0.f;
#pragma unroll
      for (int s = 0; s < KSJ; ++s) {
        const int x0 = (dsrbase[0] ^ ((s & 1) << 5) ^ (ib << 6)) + 16 * s * DSRB;
        const int x1 = (dsrbase[1] ^ ((s & 1) << 5) ^ (ib << 6)) + 16 * s * DSRB;
        const bf16x8 a = join_tr(lds_read_tr(dsb, x0), lds_read_tr(dsb, x1));
        dqacc = mfma32(a, kq[s], dqacc);
      }
      float* dst = dq_acc + head_off + dq_db * 32 + c;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = q0 + ib * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        if (i < seg_b) unsafeAtomicAdd(dst + (size_t)i * row_stride, dqacc[r]);
      }
    }
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

template <int D>
static hipError_t launch_bwd_d(const void* q, const void* k, const void* v, const void* out,
                               const float* lse, const void* dout, const SegTable& segs, int total,
                               int n_heads, float scale, void* dq, void* dk, void* dv,
                               float* dq_acc, float* delta, hipStream_t stream) {
  using Cfg = BwdCfg<D>;
  if (total == 0) return hipSuccess;
  {
    constexpr int kTokPerBlock = 256 / (D / 8);
    const int grid = (total + kTokPerBlock - 1) / kTokPerBlock;
    bwd_prepare_kernel<D><<<grid, 256, 0, stream>>>((const u32x4*)out, (const u32x4*)dout, delta,
                                                    (f32x4*)dq_acc, total, n_heads);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  int tiles = 0;
  for (int s = 0; s < segs.n; ++s) tiles += (segs.len[s] + kBwdBC - 1) / kBwdBC;
  if (tiles > 0) {
    UnitMap um;
    um.tiles_per_head = tiles;
    um.n_units = tiles * n_heads;
    um.chunk = (um.n_units + kNumXcd - 1) / kNumXcd;
    auto kern = attn_bwd_kernel<D>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    kern<<<um.chunk * kNumXcd, kBwdWaves * 64, Cfg::kLdsBytes, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)dout, lse, delta,
        (__bf16*)dk, (__bf16*)dv, dq_acc, segs, um, total, n_heads, scale, scale * kLog2eB);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  {
    const size_t n8 = (size_t)total * n_heads * D / 8;
    const unsigned grid = (unsigned)((n8 + 255) / 256);
    bwd_finish_kernel<<<grid, 256, 0, stream>>>((const f32x8*)dq_acc, (bf16x8*)dq, n8, scale);
    return hipGetLastError();
  }
}

hipError_t launch_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                           const float* lse, const void* dout, const SegTable& segs, int total,
                           int n_heads, int head_dim, float scale, void* dq, void* dk, void* dv,
                           float* dq_acc, float* delta, hipStream_t stream) {
  if (head_dim == 128)
    return launch_bwd_d<128>(q, k, v, out, lse, dout, segs, total, n_heads, scale, dq, dk, dv, dq_acc, delta, stream);
  return launch_bwd_d<64>(q, k, v, out, lse, dout, segs, total, n_heads, scale, dq, dk, dv, dq_acc, delta, stream);
}

}  // namespace vfm
