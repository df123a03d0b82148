// Packed variable-length attention forward for gfx950 (bf16 MFMA, fp32 accumulate).
//
// One workgroup owns one (head, query tile) of one clip and streams that clip's
// K/V tiles (kBC rows) through LDS, double buffered.  Each wavefront owns
// NI blocks of 32 query rows.  Scores are produced transposed,
//     S^T[j, i] = sum_d K[j, d] Q[i, d]         (32x32x16 MFMA, A = K rows, B = Q rows)
// so that a lane holds 16 key positions of ONE query row per block: the row max
// and row sum are in-lane reductions plus one exchange with lane^32, the O
// rescale is a per-lane scalar, and the bf16 P registers are already the B
// operand of
//     O^T[d, i] += sum_j V[j, d] P^T[j, i]      (A = V^T via transposing LDS reads).
// The contraction slots of that second MFMA are bound to key rows in the order the
// first MFMA's accumulator registers hold them (runs of 4 rows), which is also what
// a transposing LDS read returns, so P never leaves registers.
#include "vfm_common.h"

namespace vfm {

constexpr int kFwdWaves = 4;
constexpr int kFwdBC = 64;       // key/value rows per LDS tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleThreshold = 8.0f;  // in log2 units: lazily keep a stale row max up to 2^8

template <int D, int NI>
struct FwdCfg {
  static constexpr int kBR = kFwdWaves * NI * 32;          // query rows per workgroup
  static constexpr int kTileBytes = kFwdBC * D * 2;        // one K or V tile
  static constexpr int kLdsBytes = 4 * kTileBytes;         // K,V x 2 stages
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kChunksPerThread = kFwdBC * kChunksPerRow / (kFwdWaves * 64);
};

template <int D, int NI>
__global__ __launch_bounds__(kFwdWaves * 64, (NI == 1 ? 2 : 1))
void attn_fwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                     const __bf16* __restrict__ v, __bf16* __restrict__ out,
                     float* __restrict__ lse, const SegTable segs, const UnitMap um,
                     int total, int n_heads, float scale_log2) {
  using Cfg = FwdCfg<D, NI>;
  constexpr int KS = D / 16;   // k-steps of the QK^T contraction
  constexpr int DB = D / 32;   // 32-wide blocks of the head dimension
  constexpr int JB = kFwdBC / 32;
  constexpr int CPT = Cfg::kChunksPerThread;

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
  const size_t row_stride = (size_t)n_heads * D;   // elements between consecutive tokens
  const __bf16* kbase = k + (size_t)head * D;
  const __bf16* vbase = v + (size_t)head * D;

  // ---- Q operands (B operand of S^T): lane holds row i = c, columns ks*16 + 8g..+7
  bf16x8 qreg[NI][KS];
  int qrow[NI];
#pragma unroll
  for (int ib = 0; ib < NI; ++ib) {
    qrow[ib] = q0 + (wave * NI + ib) * 32 + c;
    const int r = min(qrow[ib], seg_b - 1);
    const __bf16* qp = q + (size_t)r * row_stride + (size_t)head * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ib][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  // ---- K/V staging with direct global->LDS loads (no staging registers, no LDS
  // writes).  One wave instruction fills 64 consecutive 16-byte chunks of a tile;
  // lane L of instruction (x, wave) owns LDS chunk P = (x*waves + wave)*64 + L, i.e.
  // tile row P / chunks_per_row, physical chunk P % chunks_per_row, and fetches the
  // logical chunk that the swizzle maps there.  Global byte offsets are 32-bit and are
  // advanced by one tile per iteration; rows past the clip end clamp to its last row.
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  const uint32_t last_row_off = (uint32_t)(seg_b - 1) * row_bytes;
  uint32_t st_rowoff[CPT], st_colb[CPT];
#pragma unroll
  for (int x = 0; x < CPT; ++x) {
    const int p = (x * kFwdWaves + wave) * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    st_rowoff[x] = (uint32_t)(seg_a + r) * row_bytes;
    st_colb[x] = (uint32_t)(((p % Cfg::kChunksPerRow) ^ swz<D>(r)) * 16);
  }
  const uint32_t smem_addr = lds_addr_of(smem);
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(smem_addr + wave * 1024);
  // issues the next tile in row order (tiles are always requested in sequence)
  auto issue_tile = [&](int stage) {
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      const uint32_t off = min(st_rowoff[x], last_row_off) + st_colb[x];
      const uint32_t dst = wave_lds + stage * 2 * Cfg::kTileBytes + x * kFwdWaves * 1024;
      lds_dma16(kbase, off, dst);
      lds_dma16(vbase, off, dst + Cfg::kTileBytes);
      st_rowoff[x] += kFwdBC * row_bytes;
    }
  };

  // ---- per-lane LDS read offsets (within a tile).  The swizzle XORs bits 4..7 of the
  // byte offset with a function of (row & 15) only, so the offsets of the other
  // k-steps / head-dim blocks / row blocks follow from one base per lane:
  //   K rows as A operand: row jb*32 + c, columns ks*16 + 8g
  //       off = (kbase ^ (ks << 5)) + jb*32*rowbytes
  //   V^T as A operand via transposing reads.  For k-step s2 of key block jb the 8
  //   contraction slots of lane group g are key rows jb*32 + 16*s2 + {4g..4g+3} (t=0)
  //   and {8+4g..8+4g+3} (t=1); the lane addresses row +((lane&15)>>2), columns
  //   db*32 + 16*((lane>>4)&1) + 4*(lane&3):
  //       off = (vbase[t] ^ (db << 6)) + (jb*32 + 16*s2)*rowbytes
  constexpr int RB = D * 2;
  const int kbase_off = tile_off<D>(c, 8 * g);
  int vbase_off[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    vbase_off[t] = tile_off<D>(8 * t + 4 * g + ((lane & 15) >> 2),
                               16 * ((lane >> 4) & 1) + 4 * (lane & 3));

  f32x16 oacc[NI][DB];
  float m_run[NI], l_run[NI];
#pragma unroll
  for (int ib = 0; ib < NI; ++ib) {
    m_run[ib] = -INFINITY;
    l_run[ib] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[ib][db][r] = 0.f;
  }

  const int n_kv = seg_b - seg_a;
  const int n_tiles = (n_kv + kFwdBC - 1) / kFwdBC;

#pragma unroll
  for (int ib = 0; ib < NI; ++ib)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) settle(qreg[ib][ks]);
  issue_tile(0);
  wait_vmcnt<0>();
  __syncthreads();

  // One tile; STAGE is a compile-time constant so every LDS offset is an immediate.
  auto tile_body = [&](auto stage_c, int t) {
    constexpr int STAGE = decltype(stage_c)::value;
    const int j0 = seg_a + t * kFwdBC;
    // the next tile's loads are issued first and land while this tile is processed
    if (t + 1 < n_tiles) issue_tile(STAGE ^ 1);

    const char* kt = smem + STAGE * 2 * Cfg::kTileBytes;
    const char* vt = kt + Cfg::kTileBytes;

    // ---- all K operand reads of this tile are issued before the first MFMA, so their
    // LDS latency overlaps; the scheduling barriers keep the compiler from
    // re-serialising read -> wait -> MFMA.
    bf16x8 ka[JB][KS];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        ka[jb][ks] = lds_read_b128(kt, (kbase_off ^ (ks << 5)) + jb * 32 * RB);
    __builtin_amdgcn_sched_barrier(0);

    // ---- S^T = K Q^T (the first k-step starts from a zero accumulator)
    f32x16 sacc[JB][NI];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int ib = 0; ib < NI; ++ib)
          sacc[jb][ib] = mfma32(ka[jb][ks], qreg[ib][ks], ks == 0 ? zero16 : sacc[jb][ib]);

    // ---- V^T operand reads are issued now, in the shadow of the S MFMAs and the softmax
    s16x4 vlo[JB][2][DB], vhi[JB][2][DB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          vlo[jb][s2][db] = lds_read_tr(vt, (vbase_off[0] ^ (db << 6)) + (jb * 32 + 16 * s2) * RB);
          vhi[jb][s2][db] = lds_read_tr(vt, (vbase_off[1] ^ (db << 6)) + (jb * 32 + 16 * s2) * RB);
        }
    __builtin_amdgcn_sched_barrier(0);

    // ---- mask keys past the end of the clip (last tile only)
    if (j0 + kFwdBC > seg_b) {
#pragma unroll
      for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + jb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (j >= seg_b) {
#pragma unroll
            for (int ib = 0; ib < NI; ++ib) sacc[jb][ib][r] = -INFINITY;
          }
        }
    }

    // ---- online softmax (log2 domain), P -> bf16
    bf16x8 pb[NI][JB][2];
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
      float mx = sacc[0][ib][0];
#pragma unroll
      for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[jb][ib][r]);
      mx = pair_max(mx) * scale_log2;
      const float m_new = fmaxf(m_run[ib], mx);
      // The reference point only moves when some row's max grew by more than the
      // threshold; otherwise exponentials are taken against the stale max (exact
      // after the final normalisation, and bounded by 2^threshold).
      if (__builtin_amdgcn_ballot_w64(m_new - m_run[ib] > kRescaleThreshold) != 0) {
        const float alpha = fast_exp2(m_run[ib] - m_new);
        l_run[ib] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[ib][db][r] *= alpha;
        m_run[ib] = m_new;
      }
      const float mref = m_run[ib];
      float lsum = 0.f;
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
        f32x8 p0, p1;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          p0[r] = fast_exp2(sacc[jb][ib][r] * scale_log2 - mref);
          p1[r] = fast_exp2(sacc[jb][ib][8 + r] * scale_log2 - mref);
          lsum += p0[r] + p1[r];
        }
        pb[ib][jb][0] = to_bf16x8(p0);
        pb[ib][jb][1] = to_bf16x8(p1);
      }
      l_run[ib] += lsum;
    }

    // ---- O^T += V^T P^T
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 va = join_tr(vlo[jb][s2][db], vhi[jb][s2][db]);
#pragma unroll
          for (int ib = 0; ib < NI; ++ib) oacc[ib][db] = mfma32(va, pb[ib][jb][s2], oacc[ib][db]);
        }
    __builtin_amdgcn_sched_barrier(0);

    wait_vmcnt<0>();   // the next tile has landed ...
    __syncthreads();   // ... for every wave, and every wave is done reading this one
  };
  for (int t = 0; t < n_tiles; t += 2) {
    tile_body(IntC<0>{}, t);
    if (t + 1 < n_tiles) tile_body(IntC<1>{}, t + 1);
  }

  // ---- epilogue: normalise, write out (bf16) and lse (natural log)
#pragma unroll
  for (int ib = 0; ib < NI; ++ib) {
    const float l_tot = pair_sum(l_run[ib]);
    const float inv = 1.0f / l_tot;
    const int i = qrow[ib];
    if (i < seg_b) {
      __bf16* op = out + (size_t)i * row_stride + (size_t)head * D + 4 * g;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = oacc[ib][db][q4 * 4 + e] * inv;
          *reinterpret_cast<bf16x4*>(op + db * 32 + q4 * 8) = to_bf16x4(o);
        }
      if (g == 0) lse[(size_t)head * total + i] = (m_run[ib] + __log2f(l_tot)) * kLn2;
    }
  }
}

template <int D, int NI>
static hipError_t launch_fwd_cfg(const void* q, const void* k, const void* v, const SegTable& segs,
                                 int total, int n_heads, float scale, void* out, float* lse,
                                 hipStream_t stream) {
  using Cfg = FwdCfg<D, NI>;
  int tiles = 0;
  for (int s = 0; s < segs.n; ++s) tiles += (segs.len[s] + Cfg::kBR - 1) / Cfg::kBR;
  if (tiles == 0) return hipSuccess;
  UnitMap um;
  um.tiles_per_head = tiles;
  um.n_units = tiles * n_heads;
  um.chunk = (um.n_units + kNumXcd - 1) / kNumXcd;
  const int grid = um.chunk * kNumXcd;
  auto kern = attn_fwd_kernel<D, NI>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
  if (e != hipSuccess) return e;
  kern<<<grid, kFwdWaves * 64, Cfg::kLdsBytes, stream>>>(
      (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (__bf16*)out, lse, segs, um, total,
      n_heads, scale * kLog2e);
  return hipGetLastError();
}

hipError_t launch_attn_fwd(const void* q, const void* k, const void* v, const SegTable& segs,
                           int total, int n_heads, int head_dim, float scale, void* out,
                           float* lse, hipStream_t stream) {
  if (head_dim == 128) return launch_fwd_cfg<128, 1>(q, k, v, segs, total, n_heads, scale, out, lse, stream);
  return launch_fwd_cfg<64, 1>(q, k, v, segs, total, n_heads, scale, out, lse, stream);
}

}  // namespace vfm
