// Packed variable-length attention forward for gfx950 (bf16 MFMA, fp32 accumulate).
//
// One workgroup (W wavefronts x 32 query rows; W = 8 at head_dim 128, two wavefronts per
// SIMD) owns one (head, query tile) of one clip and streams that clip's keys and values
// through LDS in units of 32 rows.  The more query rows share a staged unit, the fewer
// L2 -> LDS bytes move per MFMA: 256 rows instead of 128 measured 4.5% faster.
//
// Scores are produced transposed,
//     S^T[j, i] = sum_d K[j, d] Q[i, d]         (32x32x16 MFMA, A = K rows, B = Q rows)
// so that a lane holds 16 key positions of ONE query row: the row sum is an in-lane
// reduction plus one exchange with lane^32 at the end, the O rescale is a per-lane
// scalar, and the bf16 P registers are already the B operand of
//     O^T[d, i] += sum_j V[j, d] P^T[j, i]      (A = V^T via transposing LDS reads).
// The contraction slots of that second MFMA are bound to key rows in the order the first
// MFMA's accumulator registers hold them (runs of 4 rows), which is also what a
// transposing LDS read returns, so P never leaves registers.
//
// The loop is software pipelined over units so that one wavefront always has independent
// MFMA and VALU work in flight: iteration u issues the MFMAs of S(u+1) and of
// O += V(u-1) P(u-1) while the VALU computes the softmax of unit u.  A VALU instruction
// costs 4 issue cycles (exp2: ~12) against 32 for an MFMA, so about five VALU
// instructions fit under each MFMA; scheduling-group barriers ask the compiler for that
// interleave.  The softmax reference point (running max) is only moved when a unit's
// exponentials threaten to overflow, which is detected on the row sums after the fact,
// so the common path has no max reduction and no rescale.  K and V units live in two LDS rings of four slots, filled by direct
// global->LDS loads issued three units ahead.
#include "vfm_common.h"

namespace vfm {

constexpr int kFwdU = 32;               // key/value rows per pipeline unit
constexpr int kFwdRing = 4;             // LDS ring slots for K and for V
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSafeRowSum = 256.0f;  // a unit's exponentials may sum to this before the reference moves

template <int D, int W>
struct FwdCfg {
  static constexpr int kRows = W * 32;                              // query rows per workgroup
  static constexpr int kUnitBytes = kFwdU * D * 2;                  // one K or V unit
  static constexpr int kLdsBytes = 2 * kFwdRing * kUnitBytes;       // K ring + V ring
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kLoadsPerWave = kFwdU * kChunksPerRow / (W * 64);  // per unit, per tensor
};

// scheduling-group masks
constexpr int kSgValu = 0x002, kSgMfma = 0x008, kSgDsRead = 0x100;

template <int D, int W, class Segs>
__global__ __launch_bounds__(W * 64, 2)
void attn_fwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                     const __bf16* __restrict__ v, __bf16* __restrict__ out,
                     float* __restrict__ lse, const Segs segs, const UnitMap um, const TileIndex ti,
                     int total, int n_heads, float scale_log2) {
  using Cfg = FwdCfg<D, W>;
  constexpr int KS = D / 16;   // k-steps of the QK^T contraction
  constexpr int DB = D / 32;   // 32-wide blocks of the head dimension
  constexpr int LPW = Cfg::kLoadsPerWave;
  constexpr int UB = Cfg::kUnitBytes;
  constexpr int RB = D * 2;
  constexpr int kInFlight = 2 * 2 * LPW;   // loads of the two youngest batches (K and V each)

  extern __shared__ __attribute__((aligned(16))) char smem[];

  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  // query rows [q0, q0 + rows) of the sequence's query range [.., q_b); its keys and values
  // are rows [seg_a, seg_b) of k and v (the same range for self-attention)
  int seq, tq;
  locate_tile(ti, segs.n, tile, seq, tq);
  const int q_b = segs.q_start(seq) + segs.q_len(seq);
  const int q0 = segs.q_start(seq) + tq * Cfg::kRows;
  const int seg_a = segs.kv_start(seq);
  const int seg_b = seg_a + segs.kv_len(seq);

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int c = lane & 31;
  const int g = lane >> 5;
  const size_t row_stride = (size_t)n_heads * D;   // elements between consecutive tokens
  const __bf16* kbase = k + (size_t)head * D;
  const __bf16* vbase = v + (size_t)head * D;

  // ---- Q operands (B operand of S^T): lane holds row i = c, columns ks*16 + 8g..+7
  bf16x8 qreg[KS];
  const int qrow = q0 + wave * 32 + c;
  {
    const int r = min(qrow, q_b - 1);
    const __bf16* qp = q + (size_t)r * row_stride + (size_t)head * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  // ---- K/V staging with direct global->LDS loads.  One wave instruction fills 64
  // consecutive 16-byte chunks of a unit; lane L of instruction (x, wave) owns chunk
  // P = (x*waves + wave)*64 + L, i.e. unit row P / chunks_per_row, physical chunk
  // P % chunks_per_row, and fetches the logical chunk the swizzle maps there.  Global
  // byte offsets are 32-bit, advanced one unit per request; rows past the clip end clamp
  // to its last row (their scores are masked).  Units are requested strictly in order.
  const uint32_t row_bytes = (uint32_t)row_stride * 2u;
  const uint32_t last_row_off = (uint32_t)(seg_b - 1) * row_bytes;
  uint32_t st_colb[LPW], k_rowoff[LPW], v_rowoff[LPW];
#pragma unroll
  for (int x = 0; x < LPW; ++x) {
    const int p = (x * W + wave) * 64 + lane;
    const int r = p / Cfg::kChunksPerRow;
    k_rowoff[x] = v_rowoff[x] = (uint32_t)(seg_a + r) * row_bytes;
    st_colb[x] = (uint32_t)(((p % Cfg::kChunksPerRow) ^ swz<D>(r)) * 16);
  }
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(smem) + wave * 1024);
  auto issue_k = [&](int slot) {
#pragma unroll
    for (int x = 0; x < LPW; ++x) {
      lds_dma16(kbase, min(k_rowoff[x], last_row_off) + st_colb[x],
                wave_lds + slot * UB + x * W * 1024);
      k_rowoff[x] += kFwdU * row_bytes;
    }
  };
  auto issue_v = [&](int slot) {
#pragma unroll
    for (int x = 0; x < LPW; ++x) {
      lds_dma16(vbase, min(v_rowoff[x], last_row_off) + st_colb[x],
                wave_lds + (kFwdRing + slot) * UB + x * W * 1024);
      v_rowoff[x] += kFwdU * row_bytes;
    }
  };

  // ---- per-lane LDS read offsets within a unit.  The swizzle XORs bits 4..7 of the byte
  // offset with a function of (row & 15) only, so one base per lane serves every k-step
  // and head-dim block:
  //   K rows as A operand (row c, columns ks*16 + 8g):   off = kbase_off ^ (ks << 5)
  //   V^T as A operand via transposing reads.  For k-step s2 the 8 contraction slots of
  //   lane group g are key rows 16*s2 + {4g..4g+3} (t=0) and {8+4g..8+4g+3} (t=1); the
  //   lane addresses row +((lane&15)>>2), columns db*32 + 16*((lane>>4)&1) + 4*(lane&3):
  //                                                      off = (vbase_off[t] ^ (db << 6)) + 16*s2*RB
  const int kbase_off = tile_off<D>(c, 8 * g);
  int vbase_off[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
    vbase_off[t] = tile_off<D>(8 * t + 4 * g + ((lane & 15) >> 2),
                               16 * ((lane >> 4) & 1) + 4 * (lane & 3));

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) oacc[db] = zero16;

  const int n_units = (seg_b - seg_a + kFwdU - 1) / kFwdU;

  auto read_k = [&](int slot, bf16x8 (&ka)[KS]) {
    const char* kt = smem + slot * UB;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ka[ks] = lds_read_b128(kt, kbase_off ^ (ks << 5));
  };
  auto mask_tail = [&](int u, f32x16& s) {   // keys past the clip end (last unit only)
    const int j0 = seg_a + u * kFwdU;
    if (j0 + kFwdU > seg_b) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (j0 + 8 * (r >> 2) + 4 * g + (r & 3) >= seg_b) s[r] = -INFINITY;
    }
  };

  // A wavefront whose 32 query rows all lie past the end of the sequence (the ragged last
  // tile of a clip) has nothing to compute.  It still fetches its share of every K/V unit
  // and meets every barrier, in the order of the code below: the prologue's requests, wait and
  // two barriers; per unit the two requests, the
  // wait, the barrier; then the epilogue's wait and barrier.
  if (q0 + wave * 32 >= q_b) {
    issue_k(0); issue_k(1); issue_k(2); issue_k(3);
    issue_v(0); issue_v(1);
    wait_vmcnt<0>();
    __syncthreads();
    __syncthreads();
    issue_k(0);
    for (int u = 0; u < n_units; ++u) {
      issue_k((u + 1) % kFwdRing);
      issue_v((u + 2) % kFwdRing);
      wait_vmcnt<kInFlight>();
      __syncthreads();
    }
    wait_vmcnt<0>();
    __syncthreads();
    return;
  }

  // ---- prologue: K units 0..3 and V units 0..1 requested; S(0); operands of K(1)
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) settle(qreg[ks]);
  issue_k(0); issue_k(1); issue_k(2); issue_k(3);
  issue_v(0); issue_v(1);
  wait_vmcnt<0>();
  __syncthreads();

  bf16x8 ka[KS];
  f32x16 s_cur;
  {
    bf16x8 k0[KS];
    read_k(0, k0);
    read_k(1, ka);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s_cur = mfma32(k0[ks], qreg[ks], ks == 0 ? zero16 : s_cur);
    mask_tail(0, s_cur);
  }
  // the first reference point is the exact row max of unit 0, so nothing needs rescaling
  float m_run, l_run = 0.f;
  {
    float mx = s_cur[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s_cur[r]);
    m_run = pair_max(mx) * scale_log2;
  }
  __syncthreads();            // every wave holds K(0), K(1) in registers: slots 0, 1 are free
  issue_k(0);                 // K unit 4

  bf16x8 pb_prev[2];          // P(u-1), set by the first iteration before any use
  pb_prev[0] = pb_prev[1] = bf16x8{};

  // One pipeline iteration.  SLOT = u % 4 is a compile-time constant so every LDS offset
  // is an immediate.  With PV = false (u = 0) there is no previous unit to accumulate.
  auto iteration = [&](auto slot_c, auto pv_c, int u) {
    constexpr int SLOT = decltype(slot_c)::value;
    constexpr bool PV = decltype(pv_c)::value != 0;
    // requests: K(u+5) into the slot of K(u+1), V(u+2) into the slot of V(u-2)
    issue_k((SLOT + 1) % kFwdRing);
    issue_v((SLOT + 2) % kFwdRing);

    // ---- region 1: S(u+1) MFMAs | V(u-1) operand reads | first half of softmax(u)
    s16x4 vlo[2][DB], vhi[2][DB];
    if constexpr (PV) {
      const char* vt = smem + (kFwdRing + (SLOT + 3) % kFwdRing) * UB;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          vlo[s2][db] = lds_read_tr(vt, (vbase_off[0] ^ (db << 6)) + 16 * s2 * RB);
          vhi[s2][db] = lds_read_tr(vt, (vbase_off[1] ^ (db << 6)) + 16 * s2 * RB);
        }
    }
    f32x16 s_next;
    // two accumulation chains (even and odd k-steps): a single chain of dependent MFMAs
    // cannot issue back to back; the 16 extra adds cost less than the stalls they remove
    f32x16 s_odd;
#pragma unroll
    for (int ks = 0; ks < KS; ks += 2) {
      s_next = mfma32(ka[ks], qreg[ks], ks == 0 ? zero16 : s_next);
      s_odd = mfma32(ka[ks + 1], qreg[ks + 1], ks == 0 ? zero16 : s_odd);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) s_next[r] += s_odd[r];

    // softmax of unit u (log2 domain), taken against the current reference point m_run
    // without looking at this unit's maximum: the result is exact after the final
    // normalisation whatever the reference is, as long as no exponential overflows.  That
    // is checked afterwards on the row sums (see below), which costs one compare instead
    // of a max reduction per unit.
    f32x8 p0, p1;
#pragma unroll
    for (int r = 0; r < 8; ++r) p0[r] = fast_exp2(s_cur[r] * scale_log2 - m_run);
    bf16x8 pb_cur[2];
    pb_cur[0] = to_bf16x8(p0);
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) lsum += p0[r];
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kSgDsRead, PV ? 2 : 0, 0);
      __builtin_amdgcn_sched_group_barrier(kSgValu, 5, 0);
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- region 2: O += V(u-1) P(u-1) MFMAs | K(u+2) operand reads | second half of softmax(u)
    if constexpr (PV) {
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int db = 0; db < DB; ++db)
          oacc[db] = mfma32(join_tr(vlo[s2][db], vhi[s2][db]), pb_prev[s2], oacc[db]);
    }
    bf16x8 ka_next[KS];
    read_k((SLOT + 2) % kFwdRing, ka_next);
#pragma unroll
    for (int r = 0; r < 8; ++r) p1[r] = fast_exp2(s_cur[8 + r] * scale_log2 - m_run);
    pb_cur[1] = to_bf16x8(p1);
#pragma unroll
    for (int r = 0; r < 8; ++r) lsum += p1[r];
    // every P <= lsum, so a bounded sum bounds each term; an overflow (inf) fails the test too
    const bool redo = __builtin_amdgcn_ballot_w64(!(lsum <= kSafeRowSum)) != 0;
#pragma unroll
    for (int i = 0; i < 2 * DB; ++i) {
      __builtin_amdgcn_sched_group_barrier(kSgMfma, PV ? 1 : 0, 0);
      __builtin_amdgcn_sched_group_barrier(kSgDsRead, 1, 0);
      __builtin_amdgcn_sched_group_barrier(kSgValu, 4, 0);
    }
    // keep the softmax in this block: later branches must not pull it below them
    asm volatile("" : "+v"(pb_cur[0]), "+v"(pb_cur[1]), "+v"(lsum));
    __builtin_amdgcn_sched_barrier(0);

    // rare (wave-uniform): some score exceeded the reference by more than the safe margin.
    // Move the reference to the true running max, redo this unit's exponentials against
    // it and bring the sums and the accumulator (which now includes unit u-1, taken
    // against the old reference) to the new one.
    if (redo) {
      float mx = s_cur[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s_cur[r]);
      const float m_new = fmaxf(m_run, pair_max(mx) * scale_log2);
      const float alpha = fast_exp2(m_run - m_new);
      m_run = m_new;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        p0[r] = fast_exp2(s_cur[r] * scale_log2 - m_new);
        p1[r] = fast_exp2(s_cur[8 + r] * scale_log2 - m_new);
      }
      pb_cur[0] = to_bf16x8(p0);
      pb_cur[1] = to_bf16x8(p1);
      lsum = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) lsum += p0[r] + p1[r];
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    l_run += lsum;

    mask_tail(u + 1, s_next);
    s_cur = s_next;
    pb_prev[0] = pb_cur[0];
    pb_prev[1] = pb_cur[1];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ka[ks] = ka_next[ks];

    wait_vmcnt<kInFlight>();   // everything but the two youngest batches has landed ...
    __syncthreads();           // ... for every wave, and every wave is done with this unit's slots
  };

  iteration(IntC<0>{}, IntC<0>{}, 0);
  for (int u = 1; u < n_units; u += 4) {
    iteration(IntC<1>{}, IntC<1>{}, u);
    if (u + 1 < n_units) iteration(IntC<2>{}, IntC<1>{}, u + 1);
    if (u + 2 < n_units) iteration(IntC<3>{}, IntC<1>{}, u + 2);
    if (u + 3 < n_units) iteration(IntC<0>{}, IntC<1>{}, u + 3);
  }
  // ---- drain: accumulate the last unit
  {
    const char* vt = smem + (kFwdRing + (n_units - 1) % kFwdRing) * UB;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 va = join_tr(lds_read_tr(vt, (vbase_off[0] ^ (db << 6)) + 16 * s2 * RB),
                                  lds_read_tr(vt, (vbase_off[1] ^ (db << 6)) + 16 * s2 * RB));
        oacc[db] = mfma32(va, pb_prev[s2], oacc[db]);
      }
  }
  wait_vmcnt<0>();   // no load may still be writing LDS when the workgroup ends

  // ---- epilogue: normalise, write out (bf16) and lse (natural log)
  const float l_tot = pair_sum(l_run);
  const float inv = 1.0f / l_tot;
  if (qrow < q_b && g == 0) lse[(size_t)head * total + qrow] = (m_run + __log2f(l_tot)) * kLn2;
  __syncthreads();   // the rings are free: each wavefront turns its tile through a piece of them
  const int row0 = q0 + wave * 32;
  store_tile_rows<D>(smem + wave * (32 * RB), oacc, inv,
                     out + (size_t)row0 * row_stride + (size_t)head * D, row_stride, q_b - row0);
}

template <int D, int W, class Segs>
static hipError_t launch_fwd_cfg(const void* q, const void* k, const void* v, const Segs& segs,
                                 int total, int n_heads, float scale, void* out, float* lse,
                                 hipStream_t stream) {
  using Cfg = FwdCfg<D, W>;
  const TileIndex ti = make_tile_index<false>(segs, Cfg::kRows);
  const int tiles = count_tiles(ti);
  if (tiles == 0) return hipSuccess;
  UnitMap um = make_unit_map(tiles, n_heads);
  const int grid = um.chunk * kNumXcd;
  auto kern = attn_fwd_kernel<D, W, Segs>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
  if (e != hipSuccess) return e;
  return launch(kern, dim3(grid), dim3(W * 64), Cfg::kLdsBytes, stream, (const __bf16*)q, (const __bf16*)k,
                (const __bf16*)v, (__bf16*)out, lse, segs, um, ti, total, n_heads, scale * kLog2e);
}

template <class Segs>
hipError_t launch_attn_fwd(const void* q, const void* k, const void* v, const Segs& segs,
                           int total, int n_heads, int head_dim, float scale, void* out,
                           float* lse, hipStream_t stream) {
  if (head_dim == 128) {
    if (fwd_tile_rows(segs, head_dim) == 128)
      return launch_fwd_cfg<128, 4>(q, k, v, segs, total, n_heads, scale, out, lse, stream);
    return launch_fwd_cfg<128, 8>(q, k, v, segs, total, n_heads, scale, out, lse, stream);
  }
  return launch_fwd_cfg<64, 4>(q, k, v, segs, total, n_heads, scale, out, lse, stream);
}
template hipError_t launch_attn_fwd<SegTable>(const void*, const void*, const void*, const SegTable&, int,
                                              int, int, float, void*, float*, hipStream_t);
template hipError_t launch_attn_fwd<XSegTable>(const void*, const void*, const void*, const XSegTable&, int,
                                               int, int, float, void*, float*, hipStream_t);

}  // namespace vfm
