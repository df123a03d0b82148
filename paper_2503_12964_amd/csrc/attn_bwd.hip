// Packed variable-length attention backward for gfx950 (bf16 MFMA, fp32 accumulate).
//
// Three kernels, no atomics (device-wide fp32 atomics are executed at the memory side on
// this chip and were measured to bound the fused variant), so every output is written
// once and the result is bitwise reproducible:
//   bwd_prepare : Delta[h,i] = sum_d dO[i,h,d] O[i,h,d],  lse2 = lse * log2(e), and two
//                 sentinel statistics (+inf, 0) used for rows past a clip's end
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
#include <algorithm>
#include <atomic>

#include "vfm_common.h"

namespace vfm {

constexpr int kBwdWaves = 4;
constexpr int kBwdBC = 128;  // key/value rows per workgroup (32 per wavefront)
constexpr int kBwdBQ = 64;   // query rows per inner step
constexpr float kLog2eB = 1.4426950408889634f;

// ---------------------------------------------------------------- prepare
constexpr int kPrepHeads = 4;   // heads per workgroup (grid.y = ceil(n_heads / kPrepHeads))

template <int D>
__global__ __launch_bounds__(256) void bwd_prepare_kernel(const u32x4* __restrict__ out,
                                                          const u32x4* __restrict__ dout,
                                                          const float* __restrict__ lse,
                                                          float* __restrict__ delta,
                                                          float* __restrict__ lse2,
                                                          float* __restrict__ sentinel, int total,
                                                          int n_heads) {
  constexpr int kLanesPerRow = D / 8;
  constexpr int kTokPerBlock = 256 / kLanesPerRow;
  const int tok = blockIdx.x * kTokPerBlock + threadIdx.x / kLanesPerRow;
  const int chunk = threadIdx.x % kLanesPerRow;
  const bool valid = tok < total;
  const int tk = valid ? tok : total - 1;
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {   // statistics fetched for rows past a clip's end
    sentinel[0] = INFINITY;                    // lse2: P = exp2(s - inf) = 0
    sentinel[1] = 0.f;                         // Delta
  }
  // blockIdx.y picks a group of kPrepHeads heads: their rows of one token are contiguous, the
  // loads of a group are in flight together, and a small call still spreads over the chip
  const int h0 = blockIdx.y * kPrepHeads;
  u32x4 a[kPrepHeads], b[kPrepHeads];
#pragma unroll
  for (int i = 0; i < kPrepHeads; ++i) {
    const size_t row = (size_t)tk * n_heads + min(h0 + i, n_heads - 1);
    a[i] = out[row * kLanesPerRow + chunk];
    b[i] = dout[row * kLanesPerRow + chunk];
  }
#pragma unroll
  for (int i = 0; i < kPrepHeads; ++i) {
    const int h = h0 + i;
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s += __builtin_bit_cast(float, a[i][e] << 16) * __builtin_bit_cast(float, b[i][e] << 16);
      s += __builtin_bit_cast(float, a[i][e] & 0xffff0000u) * __builtin_bit_cast(float, b[i][e] & 0xffff0000u);
    }
#pragma unroll
    for (int o = kLanesPerRow / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, kLanesPerRow);
    if (valid && chunk == 0 && h < n_heads) {
      delta[(size_t)h * total + tok] = s;
      lse2[(size_t)h * total + tok] = lse[(size_t)h * total + tok] * kLog2eB;   // log2 units
    }
  }
}

// ---------------------------------------------------------------- Delta for short key ranges
// Delta_i = sum_d dO_id O_id is taken from the bf16 `out` the call is given.  In a sequence
// with a handful of keys |O| is as large as |V|, dS_ij = P_ij (dP_ij - Delta_i) is small by
// cancellation, and the rounding of `out` (2^-9 relative) shows in dQ and dK: up to 13% of the
// tensor in a two-token clip, below 0.1% from 32 keys on.  For sequences with at most
// kShortKeys keys Delta is therefore recomputed here in its other form,
//     Delta_i = sum_j P_ij dP_ij,   P_ij = exp(scale q_i.k_j - lse_i),   dP_ij = dO_i.v_j,
// in fp32 from the bf16 operands (the two forms are the same quantity for the exact O).
// One lane per query row; the key loop is uniform across the wavefront.  A negligible amount
// of work (at most 32 keys per query), launched only when the call has such a sequence.
constexpr int kShortKeys = 32;

template <int D, class Segs>
__global__ __launch_bounds__(64) void bwd_short_delta_kernel(
    const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
    const __bf16* __restrict__ dout, const float* __restrict__ lse, float* __restrict__ delta,
    const Segs segs, const TileIndex ti, int total, int n_heads, float scale) {
  int seq, t;
  locate_tile(ti, segs.n, blockIdx.x, seq, t);
  const int nk = segs.kv_len(seq);
  if (nk > kShortKeys) return;
  const int head = blockIdx.y;
  const int i = segs.q_start(seq) + t * 64 + (int)threadIdx.x;
  if (i >= segs.q_start(seq) + segs.q_len(seq)) return;
  const size_t row_stride = (size_t)n_heads * D;
  const u32x4* qi = reinterpret_cast<const u32x4*>(q + (size_t)i * row_stride + (size_t)head * D);
  const u32x4* di = reinterpret_cast<const u32x4*>(dout + (size_t)i * row_stride + (size_t)head * D);
  u32x4 qw[D / 8], dw[D / 8];     // packed bf16 pairs, widened on use
#pragma unroll
  for (int c = 0; c < D / 8; ++c) { qw[c] = qi[c]; dw[c] = di[c]; }
  const float lse_i = lse[(size_t)head * total + i];
  float acc = 0.f;
  for (int j = 0; j < nk; ++j) {
    const size_t off = (size_t)(segs.kv_start(seq) + j) * row_stride + (size_t)head * D;
    const u32x4* kj = reinterpret_cast<const u32x4*>(k + off);
    const u32x4* vj = reinterpret_cast<const u32x4*>(v + off);
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int c = 0; c < D / 8; ++c) {
      const u32x4 kw = kj[c], vw = vj[c];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s += __builtin_bit_cast(float, qw[c][e] << 16) * __builtin_bit_cast(float, kw[e] << 16);
        s += __builtin_bit_cast(float, qw[c][e] & 0xffff0000u) * __builtin_bit_cast(float, kw[e] & 0xffff0000u);
        dp += __builtin_bit_cast(float, dw[c][e] << 16) * __builtin_bit_cast(float, vw[e] << 16);
        dp += __builtin_bit_cast(float, dw[c][e] & 0xffff0000u) * __builtin_bit_cast(float, vw[e] & 0xffff0000u);
      }
    }
    acc += fast_exp2((s * scale - lse_i) * kLog2eB) * dp;
  }
  delta[(size_t)head * total + i] = acc;
}

// ---------------------------------------------------------------- dK, dV
// Software pipelined over query blocks of 32 rows so that a single wavefront per SIMD
// always has independent MFMA and VALU work: iteration b runs
//   phase A:  S(b+1), dP(b+1) MFMAs        |  P(b)  = exp2(S(b)*scale - lse2)        (VALU)
//   phase B:  dV^T += dO(b)^T P(b) MFMAs   |  dS(b) = P(b) o (dP(b) - Delta)         (VALU)
//   phase C:  dK^T += Q(b)^T dS(b) MFMAs   |  row-operand reads of block b+2, tile requests
// Q/dO tiles of 64 rows (two blocks) live in a ring of three LDS stages filled by direct
// global->LDS loads two tiles ahead; there is one workgroup barrier per tile.  (Not further
// ahead on purpose: a workgroup that runs ahead of the others of its head then waits for
// its own L2 misses while the ones behind it hit, which keeps the workgroups of an XCD on
// the same part of Q/dO; three tiles ahead was measured to quadruple the HBM fetches.)
// Query rows past the clip end need no mask: their lse2 is fetched from a +inf sentinel
// (so P = 0) and their Delta from a 0 sentinel.  Key rows past the clip end need none
// either: a lane's key only feeds that lane's own dK/dV row, which is never stored.
constexpr int kBwdRing = 3;
constexpr int kSgValuB = 0x002, kSgMfmaB = 0x008, kSgDsReadB = 0x100;

template <int D>
struct BwdCfg {
  static constexpr int kTileBytes = kBwdBQ * D * 2;                      // one Q or dO tile
  static constexpr int kStageBytes = 2 * kTileBytes;                     // Q, dO tiles of one stage
  static constexpr int kStatBytes = 4 * kBwdBQ * 4;                      // lse2, Delta (+ spare) of one stage
  // tiles first (two stages span exactly 64 KB at head_dim 128: immediate LDS offsets), statistics behind them
  static constexpr int kStatBase = kBwdRing * kStageBytes;
  static constexpr int kLdsBytes = kStatBase + kBwdRing * kStatBytes;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kLoadsPerWave = kBwdBQ * kChunksPerRow / (kBwdWaves * 64);  // per tile, per tensor
};

// SPLIT: the sequence's query range is cut into q_split chunks, one workgroup each; partial
// dK/dV are added to zeroed fp32 accumulators (dkv32: dK, then dV) with fp32 atomics and
// converted afterwards.  Used when a few long key tiles would otherwise leave CUs idle.
// The work of one workgroup: key tile tk of sequence seq, one head (and, if SPLIT, one chunk of
// the sequence's queries).
template <int D, class Segs, bool SPLIT>
__device__ __forceinline__
void bwd_dkdv_unit(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                   const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                   const float* __restrict__ lse2, const float* __restrict__ delta,
                   const float* __restrict__ sentinel,   // [+inf, 0]
                   __bf16* __restrict__ dk, __bf16* __restrict__ dv, const Segs& segs,
                   int total, int n_heads, float scale, float scale_log2,
                   float* __restrict__ dkv32, size_t kv_elems, int q_split,
                   int head, int seq, int tk, int q_chunk) {
  using Cfg = BwdCfg<D>;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int LPW = Cfg::kLoadsPerWave;
  constexpr int SB = Cfg::kStageBytes;
  constexpr int TB = Cfg::kTileBytes;
  constexpr int RB = D * 2;

  extern __shared__ __attribute__((aligned(16))) char smem[];

  // key rows [j0, j0 + kBwdBC) of the sequence's key/value range [.., kv_b); the queries it
  // walks are rows [seg_a, seg_b) of q, dout (the same range for self-attention)
  const int kv_b = segs.kv_start(seq) + segs.kv_len(seq);
  const int j0 = segs.kv_start(seq) + tk * kBwdBC;
  int qa = segs.q_start(seq), qb = qa + segs.q_len(seq);
  if constexpr (SPLIT) {   // this workgroup's share of the query tiles
    const int per = ((qb - qa + kBwdBQ - 1) / kBwdBQ + q_split - 1) / q_split * kBwdBQ;
    qa += q_chunk * per;
    qb = min(qb, qa + per);
    if (qa >= qb) return;  // nothing to add (the accumulators start at zero)
  }
  const int seg_a = qa, seg_b = qb;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int c = lane & 31;
  const int g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const size_t head_off = (size_t)head * D;

  // ---- this wavefront's key/value rows as B operands (lane: row c, columns ks*16+8g..)
  const int jrow = j0 + wave * 32 + c;
  const bool jvalid = jrow < kv_b;
  if (seg_b == seg_a) {   // keys of a sequence without queries: zero gradients (cross-attention only)
    if (jvalid) {
      u32x2 z = {0u, 0u};
#pragma unroll
      for (int x = 0; x < D / 8; ++x) {
        *reinterpret_cast<u32x2*>(dk + (size_t)jrow * row_stride + head_off + 4 * g + 8 * x) = z;
        *reinterpret_cast<u32x2*>(dv + (size_t)jrow * row_stride + head_off + 4 * g + 8 * x) = z;
      }
    }
    return;
  }
  bf16x8 kreg[KS], vreg[KS];
  {
    const size_t off = (size_t)min(jrow, kv_b - 1) * row_stride + head_off + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kreg[ks] = *reinterpret_cast<const bf16x8*>(k + off + ks * 16);
      vreg[ks] = *reinterpret_cast<const bf16x8*>(v + off + ks * 16);
    }
  }

  // ---- tile requests (direct global->LDS).  Lane L of wave instruction (x, wave) owns
  // LDS chunk P = (x*waves + wave)*64 + L of the tile (row P / chunks_per_row, physical
  // chunk P % chunks_per_row) and fetches the logical chunk the swizzle maps there.
  // Every wave also fetches 64 row statistics (4 bytes per lane): waves 0/2 lse2, waves
  // 1/3 Delta (2 and 3 into spare LDS, so that all waves have equally many loads in
  // flight).  Tiles are requested strictly in order; offsets advance by one tile.
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  const uint32_t last_row_off = (uint32_t)(seg_b - 1) * row_bytes;
  const __bf16* qbase = q + head_off;
  const __bf16* dobase = dout + head_off;
  uint32_t st_rowoff[LPW], st_colb[LPW];
#pragma unroll
  for (int x = 0; x < LPW; ++x) {
    const int p = (x * kBwdWaves + wave) * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    st_rowoff[x] = (uint32_t)(seg_a + r) * row_bytes;
    st_colb[x] = (uint32_t)(((p % Cfg::kChunksPerRow) ^ swz<D>(r)) * 16);
  }
  const bool is_lse = (wave & 1) == 0;
  const float* stat_src = uniform_ptr(is_lse ? lse2 : delta);
  const uint32_t stat_sentinel = (uint32_t)((const char*)(sentinel + (is_lse ? 0 : 1)) - (const char*)stat_src);
  int stat_row = seg_a + lane;                         // packed row this lane fetches next
  const uint32_t stat_head = (uint32_t)((size_t)head * total * 4u);
  const uint32_t smem_addr = lds_addr_of(smem);
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(smem_addr + wave * 1024);
  const uint32_t stat_lds = __builtin_amdgcn_readfirstlane(smem_addr + Cfg::kStatBase + wave * (kBwdBQ * 4));
  auto issue_tile = [&](int stage) {
#pragma unroll
    for (int x = 0; x < LPW; ++x) {
      const uint32_t off = min(st_rowoff[x], last_row_off) + st_colb[x];
      const uint32_t dst = wave_lds + stage * SB + x * kBwdWaves * 1024;
      lds_dma16(qbase, off, dst);
      lds_dma16(dobase, off, dst + TB);
      st_rowoff[x] += kBwdBQ * row_bytes;
    }
    const uint32_t soff = stat_row < seg_b ? stat_head + (uint32_t)stat_row * 4u : stat_sentinel;
    lds_dma4(stat_src, soff, stat_lds + stage * Cfg::kStatBytes);
    stat_row += kBwdBQ;
  };

  // ---- per-lane LDS offsets within a tile.  The swizzle XORs low byte-offset bits with a
  // function of the low row bits only, so one base per lane serves every k-step / block:
  //   Q/dO rows as A operand (row ib*32 + c, columns ks*16 + 8g):
  //       off = (rbase ^ (ks << 5)) + ib*32*rowbytes
  //   Q^T/dO^T as A operand through transposing reads (same slot binding as the forward
  //   kernel's V^T operand):  off = (tbase[t] ^ (db << 6)) + (ib*32 + 16*s2)*rowbytes
  const int rbase = tile_off<D>(c, 8 * g);
  int tbase[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    tbase[t] = tile_off<D>(8 * t + 4 * g + ((lane & 15) >> 2),
                           16 * ((lane >> 4) & 1) + 4 * (lane & 3));

  // Every swizzled LDS address the loop uses, held in a register of its own (made opaque so
  // that the compiler keeps them instead of recomputing them between the MFMAs): set 0 for
  // stages 0 and 1, set 1 for stage 2, whose tiles lie beyond the 64 KB an immediate reaches.
  uint32_t rb[2][KS], tb[2][2][DB];
#pragma unroll
  for (int hs = 0; hs < 2; ++hs) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      rb[hs][ks] = smem_addr + hs * 2 * SB + (rbase ^ (ks << 5));
      asm volatile("" : "+v"(rb[hs][ks]));
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tb[hs][t][db] = smem_addr + hs * 2 * SB + (tbase[t] ^ (db << 6));
        asm volatile("" : "+v"(tb[hs][t][db]));
      }
  }

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) { dkacc[db] = zero16; dvacc[db] = zero16; }

  const int n_tiles = (seg_b - seg_a + kBwdBQ - 1) / kBwdBQ;
  const int n_blocks = 2 * n_tiles;

  auto read_rows = [&](int stage, int ib, bf16x8 (&qa)[KS], bf16x8 (&da)[KS]) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint32_t a = rb[stage >> 1][ks] + (stage & 1) * SB + ib * 32 * RB;
      qa[ks] = lds_read_b128_at(a);
      da[ks] = lds_read_b128_at(a + TB);
    }
  };

  // ---- prologue: tiles 0 and 1 requested; S(0), dP(0); row operands of block 1
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) { to_agpr(kreg[ks]); to_agpr(vreg[ks]); }
  issue_tile(0); issue_tile(1);
  wait_vmcnt<0>();
  __syncthreads();

  // A wavefront whose 32 key rows all lie past the end of the sequence (ragged last tile) has
  // nothing to compute.  It still fetches its share of every Q/dO tile and meets every
  // barrier, in the order of the loop below: per tile the wait, the barrier, the request;
  // then the final wait (and the epilogue's barrier).
  if (j0 + wave * 32 >= kv_b) {
    for (int t = 0; t < n_tiles; ++t) {
      wait_vmcnt<0>();
      __syncthreads();
      issue_tile((t + 2) % kBwdRing);
    }
    wait_vmcnt<0>();
    if constexpr (!SPLIT) __syncthreads();
    return;
  }

  bf16x8 qa_n[KS], da_n[KS];      // row operands of block b+1
  f32x16 s_cur, dp_cur;           // S(b), dP(b)
  {
    bf16x8 q0r[KS], d0r[KS];
    read_rows(0, 0, q0r, d0r);
    read_rows(0, 1, qa_n, da_n);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      mfma32_v(s_cur, q0r[ks], kreg[ks], ks == 0);
      mfma32_v(dp_cur, d0r[ks], vreg[ks], ks == 0);
    }
  }

  // One pipeline iteration; POS = b % 6 fixes every LDS stage at compile time.
  auto iteration = [&](auto pos_c) {
    constexpr int POS = decltype(pos_c)::value;
    constexpr int IB = POS & 1;                          // block b within its tile
    constexpr int ST_CUR = (POS / 2) % kBwdRing;         // stage of block b's tile
    constexpr int ST_ROW = ((POS + 2) / 2) % kBwdRing;   // stage of block b+2's tile
    if constexpr (IB == 0) {
      // Start of tile t = b/2: tile t+1 must have landed for every wave before anyone reads
      // block b+2's rows, and every wave is past tile t-1, whose stage takes tile t+2.
      wait_vmcnt<0>();
      __syncthreads();
      issue_tile((ST_CUR + 2) % kBwdRing);
    }
    const float* lse_s = reinterpret_cast<const float*>(smem + Cfg::kStatBase + ST_CUR * Cfg::kStatBytes);
    const float* delta_s = lse_s + kBwdBQ;               // wave 1's statistics follow wave 0's

    // ---- phase A: S(b+1), dP(b+1) | P(b) | statistics and transposed-operand reads of block b
    // One group per MFMA, in program order (see mfma32_v): group 0 fetches lse, every group
    // two transposed operands (dO^T first: phase B needs it first), the last two Delta; the
    // 16 values of P per lane are spread over groups 2.. so that lse has arrived.
    constexpr int NG = 2 * KS;
    f32x4 l4[4], d4[4];
    s16x4 dlo[2][DB], dhi[2][DB], qlo[2][DB], qhi[2][DB];
    f32x16 s_next, dp_next, p;
    u32x8 pw;
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      const int ks = gi >> 1;
      if ((gi & 1) == 0) mfma32_v(s_next, qa_n[ks], kreg[ks], ks == 0, s_cur, p, pw);
      else mfma32_v(dp_next, da_n[ks], vreg[ks], ks == 0, s_cur, p, pw);
      if (gi == 0) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) l4[q4] = *reinterpret_cast<const f32x4*>(lse_s + IB * 32 + 8 * q4 + 4 * g);
      }
#pragma unroll
      for (int r = 2 * gi; r < 2 * gi + 2; ++r) {
        const int rr = r % (4 * DB), s2 = rr / (2 * DB), db = (rr >> 1) % DB, hi = rr & 1;
        const uint32_t o = tb[ST_CUR >> 1][hi][db] + (ST_CUR & 1) * SB + (IB * 32 + 16 * s2) * RB;
        if (r < 4 * DB) { if (hi) dhi[s2][db] = lds_read_tr_at(o + TB); else dlo[s2][db] = lds_read_tr_at(o + TB); }
        else { if (hi) qhi[s2][db] = lds_read_tr_at(o); else qlo[s2][db] = lds_read_tr_at(o); }
      }
      if (gi >= NG - 2) {
#pragma unroll
        for (int q4 = 2 * (gi - (NG - 2)); q4 < 2 * (gi - (NG - 2)) + 2; ++q4)
          d4[q4] = *reinterpret_cast<const f32x4*>(delta_s + IB * 32 + 8 * q4 + 4 * g);
      }
      // P for rows i = 8*(e/4) + 4g + e%4 of the block, column j = this lane's key; a pair
      // is converted one group after its exponentials (no transcendental-result stall)
#pragma unroll
      for (int e = 1; e < 16; e += 2)
        if (e * (NG - 2) / 16 + 3 == gi) {
          const f32x2 pr = {p[e - 1], p[e]};
          pw[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
        }
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (e * (NG - 2) / 16 + 2 == gi) p[e] = fast_exp2(s_cur[e] * scale_log2 - l4[e >> 2][e & 3]);
      __builtin_amdgcn_sched_barrier(0);
    }
    {
      const f32x2 pr = {p[14], p[15]};   // the last pair's group would be NG
      pw[7] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
    }
    bf16x8 pb[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const u32x4 w = {pw[4 * s2], pw[4 * s2 + 1], pw[4 * s2 + 2], pw[4 * s2 + 3]};
      pb[s2] = __builtin_bit_cast(bf16x8, w);
    }

    // ---- phase B: dV^T += dO(b)^T P(b) | dS(b) = P(b) o (dP(b) - Delta)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        dvacc[db] = mfma32(join_tr(dlo[s2][db], dhi[s2][db]), pb[s2], dvacc[db]);
    bf16x8 dsb[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      f32x8 a;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int r = 8 * s2 + e;
        a[e] = p[r] * (dp_cur[r] - d4[r >> 2][r & 3]);
      }
      dsb[s2] = to_bf16x8(a);
    }
#pragma unroll
    for (int i = 0; i < 2 * DB; ++i) {
      __builtin_amdgcn_sched_group_barrier(kSgMfmaB, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kSgValuB, 5, 0);
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- phase C: dK^T += Q(b)^T dS(b) | row operands of block b+2
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        dkacc[db] = mfma32(join_tr(qlo[s2][db], qhi[s2][db]), dsb[s2], dkacc[db]);
    bf16x8 qa_2[KS], da_2[KS];
    read_rows(ST_ROW, IB, qa_2, da_2);
#pragma unroll
    for (int i = 0; i < 2 * DB; ++i) {
      __builtin_amdgcn_sched_group_barrier(kSgMfmaB, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kSgDsReadB, (2 * KS + 2 * DB - 1) / (2 * DB), 0);
    }
    __builtin_amdgcn_sched_barrier(0);

    s_cur = s_next;
    dp_cur = dp_next;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) { qa_n[ks] = qa_2[ks]; da_n[ks] = da_2[ks]; }
  };

  static_assert(kBwdRing == 3, "the block loop is unrolled over the ring");
  for (int b = 0; b < n_blocks; b += 6) {
    iteration(IntC<0>{});
    iteration(IntC<1>{});
    if (b + 2 < n_blocks) { iteration(IntC<2>{}); iteration(IntC<3>{}); }
    if (b + 4 < n_blocks) { iteration(IntC<4>{}); iteration(IntC<5>{}); }
  }
  wait_vmcnt<0>();   // no load may still be writing LDS when the workgroup ends

  // ---- epilogue: dK (scaled) and dV for this lane's key row
  if (jvalid) {
    if constexpr (SPLIT) {
      float* dkp = dkv32 + ((size_t)jrow * n_heads + head) * D + 4 * g;
      float* dvp = dkp + kv_elems;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            __hip_atomic_fetch_add(dkp + db * 32 + q4 * 8 + e, dkacc[db][q4 * 4 + e] * scale, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_add(dvp + db * 32 + q4 * 8 + e, dvacc[db][q4 * 4 + e], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
          }
    }
  }
  if constexpr (!SPLIT) {
    __syncthreads();   // the ring is free: each wavefront turns its tiles through a piece of it
    char* turn = smem + wave * (32 * RB);
    const int row0 = j0 + wave * 32;
    store_tile_rows<D>(turn, dkacc, scale, dk + (size_t)row0 * row_stride + head_off, row_stride, kv_b - row0);
    store_tile_rows<D>(turn, dvacc, 1.0f, dv + (size_t)row0 * row_stride + head_off, row_stride, kv_b - row0);
  }
}

template <int D, class Segs, bool SPLIT>
__global__ __launch_bounds__(kBwdWaves * 64, 1)
void attn_bwd_dkdv_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                          const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                          const float* __restrict__ lse2, const float* __restrict__ delta,
                          const float* __restrict__ sentinel,
                          __bf16* __restrict__ dk, __bf16* __restrict__ dv,
                          const Segs segs, const UnitMap um, const TileIndex ti,
                          int total, int n_heads, float scale, float scale_log2,
                          float* __restrict__ dkv32, size_t kv_elems, int q_split) {
  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  int q_chunk = 0;
  if constexpr (SPLIT) { q_chunk = tile % q_split; tile /= q_split; }
  int seq, tk;
  locate_tile(ti, segs.n, tile, seq, tk);
  bwd_dkdv_unit<D, Segs, SPLIT>(q, k, v, dout, lse2, delta, sentinel, dk, dv, segs, total, n_heads, scale,
                                scale_log2, dkv32, kv_elems, q_split, head, seq, tk, q_chunk);
}

// fp32 accumulators -> bf16 gradients (after a split dK/dV pass); also zeroes them beforehand
__global__ void fill_zero_f32x4_kernel(f32x4* p, size_t n4) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const f32x4 z = {0.f, 0.f, 0.f, 0.f};
  if (i < n4) p[i] = z;
}
__global__ void f32_to_bf16_kernel(const f32x4* __restrict__ src, bf16x4* __restrict__ dst, size_t n4) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) dst[i] = to_bf16x4(src[i]);
}

// ---------------------------------------------------------------- dQ
constexpr int kDqBC = 64;   // key/value rows per LDS tile

template <int D, int NI, int W>
struct DqCfg {
  static constexpr int kBR = W * NI * 32;        // query rows per workgroup
  static constexpr int kTileBytes = kDqBC * D * 2;      // one K or V tile
  static constexpr int kLdsBytes = 4 * kTileBytes;      // K, V x 2 stages
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kChunksPerThread = kDqBC * kChunksPerRow / (W * 64);
};

template <int D, int NI, int W, class Segs>
__global__ __launch_bounds__(W * 64, (NI == 1 ? 2 : 1))
void attn_bwd_dq_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                        const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                        const float* __restrict__ lse2g, const float* __restrict__ delta,
                        __bf16* __restrict__ dq, const Segs segs, const UnitMap um, const TileIndex ti,
                        int total, int n_heads, float scale, float scale_log2) {
  using Cfg = DqCfg<D, NI, W>;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int JB = kDqBC / 32;
  constexpr int CPT = Cfg::kChunksPerThread;
  constexpr int RB = D * 2;

  extern __shared__ __attribute__((aligned(16))) char smem[];

  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  // query rows of the range [.., q_b); keys and values are rows [seg_a, seg_b) of k, v
  int seq, tq;
  locate_tile(ti, segs.n, tile, seq, tq);
  const int q_b = segs.q_start(seq) + segs.q_len(seq);
  const int q0 = segs.q_start(seq) + tq * Cfg::kBR;
  const int seg_a = segs.kv_start(seq);
  const int seg_b = seg_a + segs.kv_len(seq);

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
    const int r = min(qrow[ib], q_b - 1);
    const size_t off = (size_t)r * row_stride + head_off + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qreg[ib][ks] = *reinterpret_cast<const bf16x8*>(q + off + ks * 16);
      doreg[ib][ks] = *reinterpret_cast<const bf16x8*>(dout + off + ks * 16);
    }
    lse2[ib] = lse2g[(size_t)head * total + r];
    dlt[ib] = delta[(size_t)head * total + r];
  }

  // ---- K/V staging with direct global->LDS loads (same scheme as the forward kernel)
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  const uint32_t last_row_off = (uint32_t)(seg_b - 1) * row_bytes;
  uint32_t st_rowoff[CPT], st_colb[CPT];
#pragma unroll
  for (int x = 0; x < CPT; ++x) {
    const int p = (x * W + wave) * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    st_rowoff[x] = (uint32_t)(seg_a + r) * row_bytes;
    st_colb[x] = (uint32_t)(((p % Cfg::kChunksPerRow) ^ swz<D>(r)) * 16);
  }
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(smem) + wave * 1024);
  auto issue_tile = [&](int stage) {   // tiles are requested in sequence
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      const uint32_t off = min(st_rowoff[x], last_row_off) + st_colb[x];
      const uint32_t dst = wave_lds + stage * 2 * Cfg::kTileBytes + x * W * 1024;
      lds_dma16(kbase, off, dst);
      lds_dma16(vbase, off, dst + Cfg::kTileBytes);
      st_rowoff[x] += kDqBC * row_bytes;
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
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const int n_tiles = (seg_b - seg_a + kDqBC - 1) / kDqBC;
#pragma unroll
  for (int ib = 0; ib < NI; ++ib)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) { settle(qreg[ib][ks]); settle(doreg[ib][ks]); }
#pragma unroll
  for (int ib = 0; ib < NI; ++ib) asm volatile("" :: "v"(lse2[ib]), "v"(dlt[ib]));
  issue_tile(0);
  wait_vmcnt<0>();
  __syncthreads();

  auto tile_body = [&](auto stage_c, int t) {
    constexpr int STAGE = decltype(stage_c)::value;
    const int j0 = seg_a + t * kDqBC;
    if (t + 1 < n_tiles) issue_tile(STAGE ^ 1);   // lands while this tile is processed
    const char* kt = smem + STAGE * 2 * Cfg::kTileBytes;
    const char* vt = kt + Cfg::kTileBytes;
    const bool tail = (j0 + kDqBC > seg_b);

#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
      // all row operands of this key block are requested before the first MFMA
      bf16x8 ka[KS], va[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = (rbase ^ (ks << 5)) + jb * 32 * RB;
        ka[ks] = lds_read_b128(kt, off);
        va[ks] = lds_read_b128(vt, off);
      }
      __builtin_amdgcn_sched_barrier(0);
      f32x16 sacc[NI], dpacc[NI];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int ib = 0; ib < NI; ++ib) {
          sacc[ib] = mfma32(ka[ks], qreg[ib][ks], ks == 0 ? zero16 : sacc[ib]);
          dpacc[ib] = mfma32(va[ks], doreg[ib][ks], ks == 0 ? zero16 : dpacc[ib]);
        }
      // K^T operands for the dQ MFMAs, requested in the shadow of the MFMAs above
      s16x4 klo[2][DB], khi[2][DB];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          klo[s2][db] = lds_read_tr(kt, (tbase[0] ^ (db << 6)) + (jb * 32 + 16 * s2) * RB);
          khi[s2][db] = lds_read_tr(kt, (tbase[1] ^ (db << 6)) + (jb * 32 + 16 * s2) * RB);
        }
      __builtin_amdgcn_sched_barrier(0);
      bf16x8 dsb[NI][2];
#pragma unroll
      for (int ib = 0; ib < NI; ++ib) {
        f32x16 ds;
        if (tail) {   // wave-uniform: only the clip's last tile pays for the key mask
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = j0 + jb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            const float pv = (j < seg_b) ? fast_exp2(sacc[ib][r] * scale_log2 - lse2[ib]) : 0.f;
            ds[r] = pv * (dpacc[ib][r] - dlt[ib]);
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float pv = fast_exp2(sacc[ib][r] * scale_log2 - lse2[ib]);
            ds[r] = pv * (dpacc[ib][r] - dlt[ib]);
          }
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          f32x8 a;
#pragma unroll
          for (int e = 0; e < 8; ++e) a[e] = ds[8 * s2 + e];
          dsb[ib][s2] = to_bf16x8(a);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 kta = join_tr(klo[s2][db], khi[s2][db]);
#pragma unroll
          for (int ib = 0; ib < NI; ++ib) dqacc[ib][db] = mfma32(kta, dsb[ib][s2], dqacc[ib][db]);
        }
      __builtin_amdgcn_sched_barrier(0);
    }

    wait_vmcnt<0>();   // the next tile has landed ...
    __syncthreads();   // ... for every wave, and every wave is done reading this one
  };
  for (int t = 0; t < n_tiles; t += 2) {
    tile_body(IntC<0>{}, t);
    if (t + 1 < n_tiles) tile_body(IntC<1>{}, t + 1);
  }

  // ---- epilogue: dq = bf16(scale * dQ^T)
#pragma unroll
  for (int ib = 0; ib < NI; ++ib) {
    const int i = qrow[ib];
    if (i < q_b) {
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

// ---------------------------------------------------------------- dQ, 64 query rows per wavefront
// Same mathematics as attn_bwd_dq_kernel, built to halve its LDS operand traffic (under this
// chip's power limit the energy per flop is what bounds the kernels, and one LDS operand read
// per MFMA is a third of it): a wavefront owns two 32-row query blocks, so every K, V row
// operand and every K^T operand read from LDS feeds two MFMAs.  That needs 512 registers,
// i.e. one wavefront per SIMD, with the register classes chosen by hand: Q, dO rows (128) and
// the dQ^T accumulators (128) live in AGPRs, which the MFMAs address directly; S^T, dP^T and
// everything the VALU touches live in VGPRs.  All MFMAs are therefore assembly statements.
// With a single wavefront per SIMD nothing else hides the VALU work, so the two query blocks
// alternate ("half-steps"): while the VALU turns block IB's S^T, dP^T of key block b into
// dS^T, the matrix pipe runs the other block's MFMAs,
//     groups  0..15 : S^T, dP^T of the other block's next key block   (assembly, VGPR results)
//     groups 16..23 : dQ^T += K^T dS^T of the other block's previous key block
// one group per MFMA; register tuples passed through the statements (the block's S^T, so that
// nothing reads it early, and the VALU's results) pin one element of the VALU work to each group.  The compiler inserts no wait states for readers of an assembly
// MFMA's result: S^T, dP^T are read a half-step later (>= 8 MFMAs), the accumulators after
// explicit wait states at the end.
// K/V tiles of 64 keys go through a ring of three LDS stages: tile t is read from the second
// half of key block 2t-1 to the end of key block 2t+1, the workgroup meets once per tile at
// the start of key block 2t-1 (tile t landed, everybody done with tile t-2) and requests
// tile t+1 there.
constexpr int kDq2Waves = 4;
constexpr int kDq2Ring = 3;

template <int D>
struct Dq2Cfg {
  static constexpr int kBR = kDq2Waves * 64;                 // query rows per workgroup
  static constexpr int kTileBytes = kDqBC * D * 2;           // one K or V tile
  static constexpr int kStageBytes = 2 * kTileBytes;         // K tile, V tile
  static constexpr int kLdsBytes = kDq2Ring * kStageBytes;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kChunksPerThread = kDqBC * kChunksPerRow / (kDq2Waves * 64);
};

// The work of one workgroup: query tile tq of sequence seq, one head.
template <int D, class Segs>
__device__ __forceinline__
void bwd_dq2_unit(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                  const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                  const float* __restrict__ lse2g, const float* __restrict__ delta,
                  __bf16* __restrict__ dq, const Segs& segs, int total, int n_heads, float scale,
                  float scale_log2, int head, int seq, int tq) {
  using Cfg = Dq2Cfg<D>;
  constexpr int KS = D / 16;
  constexpr int DB = D / 32;
  constexpr int CPT = Cfg::kChunksPerThread;
  constexpr int RB = D * 2;
  constexpr int TB = Cfg::kTileBytes;
  constexpr int SB = Cfg::kStageBytes;
  constexpr int NG = 2 * KS + 2 * DB;   // MFMAs (groups) per half-step
  static_assert(D == 128, "tuned for head_dim 128");

  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int q_b = segs.q_start(seq) + segs.q_len(seq);
  const int q0 = segs.q_start(seq) + tq * Cfg::kBR;
  const int seg_a = segs.kv_start(seq);
  const int seg_b = seg_a + segs.kv_len(seq);

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int c = lane & 31;
  const int g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;
  const size_t head_off = (size_t)head * D;
  const __bf16* kbase = k + head_off;
  const __bf16* vbase = v + head_off;

  // ---- Q and dO rows of the two query blocks as B operands (AGPRs); lse, Delta per lane
  bf16x8 qreg[2][KS], doreg[2][KS];
  float lse2[2], dlt[2];
  int qrow[2];
#pragma unroll
  for (int ib = 0; ib < 2; ++ib) {
    qrow[ib] = q0 + (wave * 2 + ib) * 32 + c;
    const int r = min(qrow[ib], q_b - 1);
    const size_t off = (size_t)r * row_stride + head_off + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qreg[ib][ks] = *reinterpret_cast<const bf16x8*>(q + off + ks * 16);
      doreg[ib][ks] = *reinterpret_cast<const bf16x8*>(dout + off + ks * 16);
    }
    lse2[ib] = lse2g[(size_t)head * total + r];
    dlt[ib] = delta[(size_t)head * total + r];
  }

  // ---- K/V staging with direct global->LDS loads; tiles are requested in sequence
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  const uint32_t last_row_off = (uint32_t)(seg_b - 1) * row_bytes;
  uint32_t st_rowoff[CPT], st_colb[CPT];
#pragma unroll
  for (int x = 0; x < CPT; ++x) {
    const int p = (x * kDq2Waves + wave) * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    st_rowoff[x] = (uint32_t)(seg_a + r) * row_bytes;
    st_colb[x] = (uint32_t)(((p % Cfg::kChunksPerRow) ^ swz<D>(r)) * 16);
  }
  const uint32_t smem_addr = lds_addr_of(smem);
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(smem_addr + wave * 1024);
  auto issue_tile = [&](int stage) {
#pragma unroll
    for (int x = 0; x < CPT; ++x) {
      const uint32_t off = min(st_rowoff[x], last_row_off) + st_colb[x];
      const uint32_t dst = wave_lds + stage * SB + x * kDq2Waves * 1024;
      lds_dma16(kbase, off, dst);
      lds_dma16(vbase, off, dst + TB);
      st_rowoff[x] += kDqBC * row_bytes;
    }
  };

  // ---- swizzled LDS addresses, one register each (opaque, so they are kept, not recomputed)
  // (a second set for the third stage, which lies beyond the 64 KB an immediate offset
  // reaches: without it every read of that stage costs a v_add_u32, 16 per key block)
  uint32_t rb[KS], tb[2][DB], rb2[KS], tb2[2][DB];
  {
    const int rbase = tile_off<D>(c, 8 * g);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      rb[ks] = smem_addr + (rbase ^ (ks << 5));
      rb2[ks] = rb[ks] + 2 * SB;
      asm volatile("" : "+v"(rb[ks]), "+v"(rb2[ks]));
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int tbase = tile_off<D>(8 * t + 4 * g + ((lane & 15) >> 2), 16 * ((lane >> 4) & 1) + 4 * (lane & 3));
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tb[t][db] = smem_addr + (tbase ^ (db << 6));
        tb2[t][db] = tb[t][db] + 2 * SB;
        asm volatile("" : "+v"(tb[t][db]), "+v"(tb2[t][db]));
      }
    }
  }

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 dqacc[2][DB];
#pragma unroll
  for (int ib = 0; ib < 2; ++ib)
#pragma unroll
    for (int db = 0; db < DB; ++db) dqacc[ib][db] = zero16;

  const int n_tiles = (seg_b - seg_a + kDqBC - 1) / kDqBC;
  const int n_blocks = 2 * n_tiles;
  const int tail_rows = seg_b - seg_a - (n_tiles - 1) * kDqBC;   // valid rows of the last tile

#pragma unroll
  for (int ib = 0; ib < 2; ++ib)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) { to_agpr(qreg[ib][ks]); to_agpr(doreg[ib][ks]); }
#pragma unroll
  for (int ib = 0; ib < 2; ++ib) asm volatile("" :: "v"(lse2[ib]), "v"(dlt[ib]));
  // A wavefront whose 64 query rows all lie past the end of the sequence (ragged last tile)
  // has nothing to compute.  It still fetches its share of every K/V tile, takes part in
  // zeroing the last tile's tail rows and meets every barrier, in the order of the loop
  // below: the prologue's requests, wait and barrier; from the second tile on the wait, the
  // barrier, the request; the two barriers
  // around the zeroing; the epilogue's wait and barrier.
  if (q0 + wave * 64 >= q_b) {
    issue_tile(0);
    issue_tile(1);
    wait_vmcnt<2 * CPT>();
    __syncthreads();
    for (int t = 1; t < n_tiles; ++t) {
      wait_vmcnt<0>();
      __syncthreads();
      if (t + 1 < n_tiles) issue_tile((t + 1) % kDq2Ring);
    }
    if (tail_rows < kDqBC) {
      __syncthreads();
      const u32x4 z = {0u, 0u, 0u, 0u};
      const int n16 = (kDqBC - tail_rows) * (RB / 16);
      for (int i = tid; i < n16; i += kDq2Waves * 64)
        *reinterpret_cast<__attribute__((address_space(3))) u32x4*>(
            smem_addr + ((n_tiles - 1) % kDq2Ring) * SB + tail_rows * RB + i * 16) = z;
      __syncthreads();
    }
    wait_vmcnt<0>();
    __syncthreads();
    return;
  }

  issue_tile(0);
  issue_tile(1);              // (re-requests the last rows when the clip has a single tile)
  wait_vmcnt<2 * CPT>();      // tile 0 has landed
  __syncthreads();

  // ---- state carried between half-steps
  f32x16 sacc[2], dpacc[2];   // S^T, dP^T of the current key block, per query block
  f32x16 dsf;                 // dS^T of the half-step at hand, fp32
  u32x8 pw[2];                // dS^T as bf16 pairs, per query block: B operands of the update
  bf16x8 ka[KS], va[KS];      // row operands of the key block whose scores come next
  s16x4 klo[2][DB], khi[2][DB];   // K^T operands of the key block whose update comes next
#pragma unroll
  for (int i = 0; i < 8; ++i) { pw[0][i] = 0u; pw[1][i] = 0u; }
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
    for (int db = 0; db < DB; ++db) { klo[s2][db] = s16x4{0, 0, 0, 0}; khi[s2][db] = s16x4{0, 0, 0, 0}; }
  dsf = zero16;

  // prologue: row operands of key block 0, S^T and dP^T of (key block 0, query block 0)
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    ka[ks] = lds_read_b128_at(rb[ks]);
    va[ks] = lds_read_b128_at(rb[ks] + TB);
  }
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    mfma32_v(sacc[0], ka[ks], qreg[0][ks], ks == 0);
    mfma32_v(dpacc[0], va[ks], doreg[0][ks], ks == 0);
  }
  sacc[1] = zero16;
  dpacc[1] = zero16;

  // One half-step.  POSB = b % 6 fixes every LDS stage at compile time; IB is the query block
  // whose dS^T the VALU forms.
  auto half_step = [&](auto posb_c, auto ib_c, int b) {
    constexpr int POSB = decltype(posb_c)::value;
    constexpr int IB = decltype(ib_c)::value;
    constexpr int OB = 1 - IB;                               // the block the matrix pipe works for
    constexpr int ST_CUR = (POSB / 2) % kDq2Ring;            // stage of key block b
    constexpr int ST_NEXT = ((POSB + 1) / 2) % kDq2Ring;     // stage of key block b+1
    constexpr int JB_CUR = POSB & 1, JB_NEXT = (POSB + 1) & 1;
    const float lse_i = lse2[IB];
    // Delta is made a new value here: the subtractions dP - Delta then cannot be moved up into the
    // previous half-step, where the MFMAs that produce dP are still running (dP itself is not
    // passed through the statements)
    float dlt_i = dlt[IB];
    asm volatile("" : "+v"(dlt_i));
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
      // ---- matrix pipe
      if (gi < 2 * KS) {
        const int ks = gi >> 1;
        if ((gi & 1) == 0) mfma32_v(sacc[OB], ka[ks], qreg[OB][ks], ks == 0, sacc[IB], dsf, pw[IB]);
        else mfma32_v(dpacc[OB], va[ks], doreg[OB][ks], ks == 0, sacc[IB], dsf, pw[IB]);
      } else {
        const int s2 = (gi - 2 * KS) / DB, db = (gi - 2 * KS) % DB;
        const u32x4 w = {pw[OB][4 * s2], pw[OB][4 * s2 + 1], pw[OB][4 * s2 + 2], pw[OB][4 * s2 + 3]};
        mfma32_acc(dqacc[OB][db], join_tr(klo[s2][db], khi[s2][db]), __builtin_bit_cast(bf16x8, w),
                   sacc[IB], dsf, pw[IB]);
      }
      // ---- LDS reads
      if (IB == 0) {
        // row operands of key block b+1, once the score MFMAs have consumed those of block b
        if (gi >= 2 * KS) {
          constexpr int per = (2 * KS) / (2 * DB);   // reads per group: 16 / 8
#pragma unroll
          for (int x = (gi - 2 * KS) * per; x < (gi - 2 * KS + 1) * per; ++x) {
            const int ks = x >> 1;
            const uint32_t a = (ST_NEXT == 2 ? rb2[ks] : rb[ks] + ST_NEXT * SB) + JB_NEXT * 32 * RB;
            if ((x & 1) == 0) ka[ks] = lds_read_b128_at(a); else va[ks] = lds_read_b128_at(a + TB);
          }
        }
      } else {
        // K^T operands of key block b (the updates of block b-1 were all issued a half-step ago)
        if (gi < 2 * DB) {
#pragma unroll
          for (int x = 2 * gi; x < 2 * gi + 2; ++x) {
            const int s2 = x / (2 * DB), db = (x >> 1) % DB, hi = x & 1;
            const uint32_t a = (ST_CUR == 2 ? tb2[hi][db] : tb[hi][db] + ST_CUR * SB) + (JB_CUR * 32 + 16 * s2) * RB;
            if (hi) khi[s2][db] = lds_read_tr_at(a); else klo[s2][db] = lds_read_tr_at(a);
          }
        }
      }
      // ---- VALU: one element of dS^T per group (keys i = 8*(e/4) + 4g + e%4 of the block, this
      // lane's query row): the exponential in group G(e), the product one group later (no
      // stall on the transcendental's result), the conversion of a pair one group after that
#pragma unroll
      for (int e = 1; e < 16; e += 2)
        if (1 + e * (NG - 2) / 16 + 2 == gi) {
          const f32x2 pr = {dsf[e - 1], dsf[e]};
          pw[IB][e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
        }
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (1 + e * (NG - 2) / 16 + 1 == gi) dsf[e] = dsf[e] * (dpacc[IB][e] - dlt_i);
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (1 + e * (NG - 2) / 16 == gi) dsf[e] = fast_exp2(sacc[IB][e] * scale_log2 - lse_i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto block = [&](auto posb_c, int b) {
    constexpr int POSB = decltype(posb_c)::value;
    if constexpr ((POSB & 1) == 1) {
      // key block 2t-1: tile t has landed for every wave, every wave is done with tile t-2,
      // whose stage takes tile t+1
      const int t = (b + 1) >> 1;
      if (t < n_tiles) {
        wait_vmcnt<0>();
        __syncthreads();
        if (t + 1 < n_tiles) issue_tile(((POSB + 1) / 2 + 1) % kDq2Ring);
      }
    }
    half_step(posb_c, IntC<0>{}, b);
    if constexpr ((POSB & 1) == 0) {
      // Keys past the clip's end (last tile only).  Their K, V rows were fetched as copies of
      // the last valid row, so their S^T, dP^T are finite and so is dS^T; what keeps them out
      // of dQ is a zero K^T column.  All row reads of this tile have been issued by now and
      // its first K^T read follows: zero those K rows in LDS in between.
      if (b == n_blocks - 2 && tail_rows < kDqBC) {
        __syncthreads();
        const u32x4 z = {0u, 0u, 0u, 0u};
        const int n16 = (kDqBC - tail_rows) * (RB / 16);
        for (int i = tid; i < n16; i += kDq2Waves * 64)
          *reinterpret_cast<__attribute__((address_space(3))) u32x4*>(
              smem_addr + ((POSB / 2) % kDq2Ring) * SB + tail_rows * RB + i * 16) = z;
        __syncthreads();
      }
    }
    half_step(posb_c, IntC<1>{}, b);
  };
  for (int b = 0; b < n_blocks; b += 6) {
    block(IntC<0>{}, b);
    block(IntC<1>{}, b + 1);
    if (b + 2 < n_blocks) { block(IntC<2>{}, b + 2); block(IntC<3>{}, b + 3); }
    if (b + 4 < n_blocks) { block(IntC<4>{}, b + 4); block(IntC<5>{}, b + 5); }
  }
  // drain: the last key block's update for query block 1
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const u32x4 w = {pw[1][4 * s2], pw[1][4 * s2 + 1], pw[1][4 * s2 + 2], pw[1][4 * s2 + 3]};
      mfma32_acc(dqacc[1][db], join_tr(klo[s2][db], khi[s2][db]), __builtin_bit_cast(bf16x8, w));
    }
  wait_vmcnt<0>();   // no load may still be writing LDS when the workgroup ends
  // the accumulators were written by assembly: wait out the last MFMA before they are read
#pragma unroll
  for (int ib = 0; ib < 2; ++ib) wait_mfma_a(dqacc[ib][0], dqacc[ib][1], dqacc[ib][2], dqacc[ib][3]);

  // ---- epilogue: dq = bf16(scale * dQ^T), whole rows per store
  __syncthreads();   // the ring is free: each wavefront turns its tiles through a piece of it
#pragma unroll
  for (int ib = 0; ib < 2; ++ib) {
    const int row0 = q0 + (wave * 2 + ib) * 32;
    store_tile_rows<D>(smem + wave * (32 * D * 2), dqacc[ib], scale,
                       dq + (size_t)row0 * row_stride + head_off, row_stride, q_b - row0);
  }
}

template <int D, class Segs>
__global__ __launch_bounds__(kDq2Waves * 64, 1)
void attn_bwd_dq2_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                         const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                         const float* __restrict__ lse2g, const float* __restrict__ delta,
                         __bf16* __restrict__ dq, const Segs segs, const UnitMap um, const TileIndex ti,
                         int total, int n_heads, float scale, float scale_log2) {
  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  int seq, tq;
  locate_tile(ti, segs.n, tile, seq, tq);
  bwd_dq2_unit<D, Segs>(q, k, v, dout, lse2g, delta, dq, segs, total, n_heads, scale, scale_log2, head, seq, tq);
}

// ---------------------------------------------------------------- short sequences: one launch
// For sequences of a few hundred tokens the two passes above are bound by the memory path, not
// by the matrix pipe: each reads q, k, v, dout of a (sequence, head) once, a millisecond apart,
// so the second pass finds nothing of it in L2.  This kernel runs the same two units from one
// grid: per (head, sequence) the key tiles' dK/dV units, then the query tiles' dQ units, as
// consecutive workgroups of one XCD, so that they run side by side and share the lines they
// fetch.  ti counts both kinds of tile per sequence (key tiles first).
template <int D, class Segs>
__global__ __launch_bounds__(kBwdWaves * 64, 1)
void attn_bwd_both_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                          const __bf16* __restrict__ v, const __bf16* __restrict__ dout,
                          const float* __restrict__ lse2, const float* __restrict__ delta,
                          const float* __restrict__ sentinel, __bf16* __restrict__ dq,
                          __bf16* __restrict__ dk, __bf16* __restrict__ dv,
                          const Segs segs, const UnitMap um, const TileIndex ti,
                          int total, int n_heads, float scale, float scale_log2) {
  static_assert(kBwdWaves == kDq2Waves, "one workgroup shape for both units");
  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  int seq, t;
  locate_tile(ti, segs.n, tile, seq, t);
  const int key_tiles = (segs.kv_len(seq) + kBwdBC - 1) / kBwdBC;
  if (t < key_tiles)
    bwd_dkdv_unit<D, Segs, false>(q, k, v, dout, lse2, delta, sentinel, dk, dv, segs, total, n_heads, scale,
                                  scale_log2, nullptr, 0, 1, head, seq, t, 0);
  else
    bwd_dq2_unit<D, Segs>(q, k, v, dout, lse2, delta, dq, segs, total, n_heads, scale, scale_log2, head, seq,
                          t - key_tiles);
}

// Sequences up to this many rows (queries and keys) take the single launch above.
constexpr int kBothMaxRows = 1024;

// Compute units of the current device (asked once; 256 on MI355X, also the fallback).
static int compute_unit_count() {
  static std::atomic<int> cached{0};
  int n = cached.load(std::memory_order_relaxed);
  if (n > 0) return n;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
    n = 256;
  cached.store(n, std::memory_order_relaxed);
  return n;
}

template <int D, class Segs>
static hipError_t launch_bwd_d(const void* q, const void* k, const void* v, const void* out,
                               const float* lse, const void* dout, const Segs& segs, int total,
                               int n_heads, float scale, void* dq, void* dk, void* dv,
                               float* delta, float* lse2, float* sentinel, float* dkv32, int total_kv,
                               int kv_lo, int kv_hi, hipStream_t stream) {
  const __bf16 *qb = (const __bf16*)q, *kb = (const __bf16*)k, *vb = (const __bf16*)v, *dob = (const __bf16*)dout;
  hipError_t e;
  if (total > 0) {   // (with no queries at all only the keys' zero gradients remain to be written)
    bool any_short = false;
    for (int s2 = 0; s2 < segs.n; ++s2)
      any_short |= segs.q_len(s2) > 0 && segs.kv_len(s2) > 0 && segs.kv_len(s2) <= kShortKeys;
    if (any_short) {   // sequences with a handful of keys: Delta in its cancellation-free form
      const TileIndex ti = make_tile_index<false>(segs, 64);
      e = launch(bwd_short_delta_kernel<D, Segs>, dim3(count_tiles(ti), n_heads), dim3(64), 0,
                 stream, qb, kb, vb, dob, lse, delta, segs, ti, total, n_heads, scale);
      if (e != hipSuccess) return e;
    }
  }
  {
    using Cfg = BwdCfg<D>;
    const TileIndex ti = make_tile_index<true>(segs, kBwdBC);
    const int tiles = count_tiles(ti);
    if (tiles == 0) return hipSuccess;
    UnitMap um = make_unit_map(tiles, n_heads);
    // Few key tiles and long query ranges (cross-attention): split the queries over workgroups.
    int q_split = 1;
    const int cus = compute_unit_count();
    if (dkv32 && tiles * n_heads < cus) {
      int max_q = 0;
      for (int s2 = 0; s2 < segs.n; ++s2) max_q = std::max(max_q, segs.q_len(s2));
      q_split = std::min(std::min(16, (cus + tiles * n_heads - 1) / (tiles * n_heads)), std::max(1, max_q / 512));
    }
    if constexpr (D == 128) {
      int longest = 0;
      for (int s2 = 0; s2 < segs.n; ++s2) longest = std::max(longest, std::max(segs.q_len(s2), segs.kv_len(s2)));
      if (q_split == 1 && longest <= kBothMaxRows) {   // short sequences: both passes from one grid
        TileIndex both;
        int n_both = 0;
        for (int s2 = 0; s2 <= VFM_MAX_SEQS; ++s2) {
          both.cu[s2] = n_both;
          if (s2 < segs.n)
            n_both += (segs.kv_len(s2) + kBwdBC - 1) / kBwdBC + (segs.q_len(s2) + Dq2Cfg<D>::kBR - 1) / Dq2Cfg<D>::kBR;
        }
        um = make_unit_map(n_both, n_heads);
        constexpr int lds = Cfg::kLdsBytes > Dq2Cfg<D>::kLdsBytes ? Cfg::kLdsBytes : Dq2Cfg<D>::kLdsBytes;
        auto kern = attn_bwd_both_kernel<D, Segs>;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        return launch(kern, dim3(um.chunk * kNumXcd), dim3(kBwdWaves * 64), lds, stream, qb, kb, vb, dob, lse2,
                      delta, sentinel, (__bf16*)dq, (__bf16*)dk, (__bf16*)dv, segs, um, both, total, n_heads, scale,
                      scale * kLog2eB);
      }
    }
    if (q_split > 1) {
      // the accumulators and the conversion cover this run's key rows [kv_lo, kv_hi) only:
      // other runs of the same call own the rest of dk, dv
      const size_t kv_elems = (size_t)total_kv * n_heads * D;
      const size_t lo4 = (size_t)kv_lo * n_heads * D / 4, h4 = (size_t)(kv_hi - kv_lo) * n_heads * D / 4;
      const dim3 cgrid((unsigned)((h4 + 255) / 256));
      f32x4* acc_k = (f32x4*)dkv32 + lo4;
      f32x4* acc_v = (f32x4*)(dkv32 + kv_elems) + lo4;
      e = launch(fill_zero_f32x4_kernel, cgrid, dim3(256), 0, stream, acc_k, h4);
      if (e != hipSuccess) return e;
      e = launch(fill_zero_f32x4_kernel, cgrid, dim3(256), 0, stream, acc_v, h4);
      if (e != hipSuccess) return e;
      um = make_unit_map(tiles * q_split, n_heads);
      auto kern = attn_bwd_dkdv_kernel<D, Segs, true>;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
      if (e != hipSuccess) return e;
      e = launch(kern, dim3(um.chunk * kNumXcd), dim3(kBwdWaves * 64), Cfg::kLdsBytes, stream, qb, kb, vb, dob,
                 lse2, delta, sentinel, (__bf16*)dk, (__bf16*)dv, segs, um, ti, total, n_heads, scale,
                 scale * kLog2eB, dkv32, kv_elems, q_split);
      if (e != hipSuccess) return e;
      e = launch(f32_to_bf16_kernel, cgrid, dim3(256), 0, stream, (const f32x4*)acc_k, (bf16x4*)dk + lo4, h4);
      if (e != hipSuccess) return e;
      e = launch(f32_to_bf16_kernel, cgrid, dim3(256), 0, stream, (const f32x4*)acc_v, (bf16x4*)dv + lo4, h4);
      if (e != hipSuccess) return e;
    } else {
      auto kern = attn_bwd_dkdv_kernel<D, Segs, false>;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
      if (e != hipSuccess) return e;
      e = launch(kern, dim3(um.chunk * kNumXcd), dim3(kBwdWaves * 64), Cfg::kLdsBytes, stream, qb, kb, vb, dob,
                 lse2, delta, sentinel, (__bf16*)dk, (__bf16*)dv, segs, um, ti, total, n_heads, scale,
                 scale * kLog2eB, (float*)nullptr, (size_t)0, 1);
      if (e != hipSuccess) return e;
    }
  }
  if constexpr (D == 128) {
    using Cfg = Dq2Cfg<D>;
    const TileIndex ti = make_tile_index<false>(segs, Cfg::kBR);
    const int tiles = count_tiles(ti);
    if (tiles == 0) return hipSuccess;
    UnitMap um = make_unit_map(tiles, n_heads);
    auto kern = attn_bwd_dq2_kernel<D, Segs>;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    return launch(kern, dim3(um.chunk * kNumXcd), dim3(kDq2Waves * 64), Cfg::kLdsBytes, stream, qb, kb, vb, dob,
                  lse2, delta, (__bf16*)dq, segs, um, ti, total, n_heads, scale, scale * kLog2eB);
  } else {
    constexpr int NI = 1;
    constexpr int W = 8;   // 256 query rows share each staged K/V tile
    using Cfg = DqCfg<D, NI, W>;
    const TileIndex ti = make_tile_index<false>(segs, Cfg::kBR);
    const int tiles = count_tiles(ti);
    if (tiles == 0) return hipSuccess;
    UnitMap um = make_unit_map(tiles, n_heads);
    auto kern = attn_bwd_dq_kernel<D, NI, W, Segs>;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    return launch(kern, dim3(um.chunk * kNumXcd), dim3(W * 64), Cfg::kLdsBytes, stream, qb, kb, vb, dob, lse2,
                  delta, (__bf16*)dq, segs, um, ti, total, n_heads, scale, scale * kLog2eB);
  }
}

// Delta, lse in log2 units and the sentinels for all `total` query tokens of a call (once per
// call, before the runs of clips).
hipError_t launch_bwd_prepare(const void* out, const void* dout, const float* lse, float* delta, float* lse2,
                              float* sentinel, int total, int n_heads, int head_dim, hipStream_t stream) {
  if (total == 0) return hipSuccess;
  const int tok_per_block = 256 / (head_dim / 8);
  const dim3 grid((total + tok_per_block - 1) / tok_per_block, (n_heads + kPrepHeads - 1) / kPrepHeads);
  if (head_dim == 128)
    return launch(bwd_prepare_kernel<128>, grid, dim3(256), 0, stream, (const u32x4*)out, (const u32x4*)dout, lse,
                  delta, lse2, sentinel, total, n_heads);
  return launch(bwd_prepare_kernel<64>, grid, dim3(256), 0, stream, (const u32x4*)out, (const u32x4*)dout, lse,
                delta, lse2, sentinel, total, n_heads);
}

template <class Segs>
hipError_t launch_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                           const float* lse, const void* dout, const Segs& segs, int total,
                           int n_heads, int head_dim, float scale, void* dq, void* dk, void* dv,
                           float* delta, float* lse2, float* sentinel, float* dkv32, int total_kv,
                           int kv_lo, int kv_hi, hipStream_t stream) {
  if (head_dim == 128)
    return launch_bwd_d<128>(q, k, v, out, lse, dout, segs, total, n_heads, scale, dq, dk, dv, delta, lse2, sentinel, dkv32, total_kv, kv_lo, kv_hi, stream);
  return launch_bwd_d<64>(q, k, v, out, lse, dout, segs, total, n_heads, scale, dq, dk, dv, delta, lse2, sentinel, dkv32, total_kv, kv_lo, kv_hi, stream);
}
template hipError_t launch_attn_bwd<SegTable>(const void*, const void*, const void*, const void*, const float*,
                                              const void*, const SegTable&, int, int, int, float, void*, void*,
                                              void*, float*, float*, float*, float*, int, int, int, hipStream_t);
template hipError_t launch_attn_bwd<XSegTable>(const void*, const void*, const void*, const void*, const float*,
                                               const void*, const XSegTable&, int, int, int, float, void*, void*,
                                               void*, float*, float*, float*, float*, int, int, int, hipStream_t);

}  // namespace vfm
