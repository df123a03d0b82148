// FP8 (E4M3) attention forward for gfx950, and the packing pass that prepares its operands.
//
// v_mfma_f32_32x32x64_f8f6f4 contracts 64 fp8 values per instruction (a lane holds 32 bytes of
// one operand row) at about twice the bf16 rate, so the kernel works in units of 64 keys:
//     S^T[64 keys, 32 q] = K Q^T      two 32-key tiles x (D/64) instructions, A = K rows, B = Q rows
//     O^T[D, 32 q]      += V^T P^T    D/32 instructions, A = rows of V^T, B = P (fp8) from registers
// The contraction slots of the second product are bound to keys in the order the first
// product's accumulators hold them, as in the bf16 kernel; here that order is baked into the
// packed V^T buffer, so each lane's 32 keys are 32 contiguous bytes.
//
// Packed operand layout (written by vfm_fp8_pack, all fp8 bytes, per head h):
//   q8  [H][total][D]                       plain rows
//   scales: [H][total] bytes (127 - e of each q row), padded to 256 bytes, then [H][units] 32-bit
//           words (byte 0: 127 - e of the k unit, byte 1: 127 - e of the v unit, bytes 2, 3: 127)
//   k8  [H][units][64 keys][D]              one unit = 64 consecutive keys of ONE clip (zero padded
//   vT8 [H][units][D][64 keys, permuted]    at the clip's end), contiguous, with the LDS bank
//                                           swizzle already applied to its 16-byte chunks
// so a unit is staged by a linear 8 KB (D = 128) direct-to-LDS copy with no address arithmetic,
// and both operand reads are conflict-free 16-byte LDS reads.
//
// Per-tile scales.  Every tile is stored as the E4M3 codes of x * 2^e with its own exponent e, the
// largest with max|x| * 2^e <= 448: one e per (token, head) row of q (which also carries
// scale * log2(e), so that q8 . k8 is the softmax exponent in log2 units), one per (head, unit)
// of k and one per (head, unit) of v.  The matrix instruction takes a power-of-two block scale
// for each lane's 32 operand bytes, so the descaling 2^-e costs nothing: the score
// instruction gets the unit's k scale and the lane's q-row scale, the second product the
// unit's v scale.  (Checked on the GPU first: lane l's scale byte applies to the 32 operand
// bytes lane l supplies, and the op-sel field picks the byte of the scale register.)  The scale
// bytes of a unit's k and v travel with the unit: one wavefront lane copies the unit's 4-byte
// scale word into a ring slot beside the unit's tiles with the same direct-to-LDS load.
// P is scaled per query row by the softmax reference point, plus a fixed 2^6:
//
// Softmax as in the bf16 kernel (lazy reference point, overflow detected on the row sums),
// except that the exponentials are scaled by 2^6 before they are rounded to E4M3, which keeps
// small probabilities out of the subnormal range (P <= 448 * 2^-6 = 7 relative to the reference).
#include "vfm_common.h"

namespace vfm {

namespace {

constexpr int kF8Unit = 64;
constexpr int kF8Waves = 8;
constexpr int kF8Rows = kF8Waves * 32;   // query rows per workgroup
constexpr int kF8Ring = 4;
constexpr float kF8Ln2 = 0.6931471805599453f;
constexpr float kF8PShift = 6.0f;        // P is stored as 2^6 P
constexpr float kF8SafeSum = 448.0f;     // largest finite E4M3: bounds every scaled P of the unit
constexpr float kF8Max = 448.0f;

typedef int i32x8 __attribute__((ext_vector_type(8)));

// LDS / packed-buffer swizzle of the 16-byte chunk index
template <int D>
__device__ __host__ __forceinline__ int k_swz(int key_row) {      // K unit: rows of D bytes
  return D == 128 ? ((key_row >> 1) & 7) : ((key_row >> 2) & 3);
}
__device__ __host__ __forceinline__ int v_swz(int d_row) { return (d_row >> 2) & 3; }   // V^T unit: rows of 64 bytes

__device__ __forceinline__ float clamp448(float x) { return fminf(fmaxf(x, -kF8Max), kF8Max); }

// four floats -> four E4M3 bytes (round to nearest even; the inputs are already within +-448)
__device__ __forceinline__ uint32_t pack_fp8x4(float a, float b, float c, float d) {
  // (the first conversion's "old" word is overwritten by the second: any register will do)
  int v = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, __builtin_bit_cast(int, a), false);
  v = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, v, true);
  return (uint32_t)v;
}

// 16 bf16 values (two 16-byte words) -> 16 E4M3 bytes of (x * pre) * pow2, clamped to +-448.
// (x * pre) is rounded to fp32 once; the power of two is exact.
__device__ __forceinline__ u32x4 quantize16(u32x4 lo, u32x4 hi, float pre, float pow2) {
  u32x4 o;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const u32x4& src = w < 2 ? lo : hi;
    const uint32_t a = src[(2 * w) & 3], b = src[(2 * w + 1) & 3];
    o[w] = pack_fp8x4(clamp448((__builtin_bit_cast(float, a << 16) * pre) * pow2),
                      clamp448((__builtin_bit_cast(float, a & 0xffff0000u) * pre) * pow2),
                      clamp448((__builtin_bit_cast(float, b << 16) * pre) * pow2),
                      clamp448((__builtin_bit_cast(float, b & 0xffff0000u) * pre) * pow2));
  }
  return o;
}

// largest |x * pre| of the same 16 values
__device__ __forceinline__ float amax16(u32x4 lo, u32x4 hi, float pre) {
  float m = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    m = fmaxf(m, fabsf(__builtin_bit_cast(float, lo[w] << 16) * pre));
    m = fmaxf(m, fabsf(__builtin_bit_cast(float, lo[w] & 0xffff0000u) * pre));
    m = fmaxf(m, fabsf(__builtin_bit_cast(float, hi[w] << 16) * pre));
    m = fmaxf(m, fabsf(__builtin_bit_cast(float, hi[w] & 0xffff0000u) * pre));
  }
  return m;
}

// Scale exponent of a tile whose largest magnitude is amax: the largest e with amax * 2^e <= 448
// (= 1.75 * 2^8), from the bits of amax; limited to [-120, 120]; 0 for an all-zero tile.
__device__ __forceinline__ int tile_exponent(float amax) {
  const uint32_t u = __builtin_bit_cast(uint32_t, amax);
  if (u == 0u) return 0;
  const int ex = (int)((u >> 23) & 0xffu) - 127;          // amax = (1 + mant / 2^23) * 2^ex  (a denormal reads as 2^-127)
  const int e = 8 - ex - ((u & 0x7fffffu) > 0x600000u ? 1 : 0);
  return min(120, max(-120, e));
}
__device__ __forceinline__ float pow2f(int e) { return __builtin_bit_cast(float, (uint32_t)(e + 127) << 23); }

// formats 0/0 = E4M3 for both operands; sa, sb: block-scale registers (an 8-bit exponent, bias 127,
// in the byte OA / OB selects) applied to the 32 bytes this lane supplies of a and of b
template <int OA, int OB>
__device__ __forceinline__ f32x16 mfma_f8(i32x8 a, i32x8 b, f32x16 c, int sa, int sb) {
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, OA, sa, OB, sb);
}
constexpr int kScaleOne = 0x7f7f7f7f;    // 2^0 in every byte

__device__ __forceinline__ i32x8 lds_read_32b(const char* base, int off0, int off1) {
  const u32x4 lo = *reinterpret_cast<const u32x4*>(base + off0);
  const u32x4 hi = *reinterpret_cast<const u32x4*>(base + off1);
  i32x8 r = {(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
  return r;
}

}  // namespace

// ---------------------------------------------------------------- packing
// q: D/16 lanes per (token, head) row, one 16-byte output chunk each; the row's largest magnitude is
// reduced over those lanes.
template <int D>
__global__ __launch_bounds__(256) void fp8_pack_q_kernel(const u32x4* __restrict__ q,
                                                         u32x4* __restrict__ q8,
                                                         unsigned char* __restrict__ q_exp, float pre,
                                                         int total, int n_heads) {
  constexpr int CPR = D / 16;   // 16-byte output chunks per row
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long n_rows = (long long)total * n_heads;
  const int chunk = (int)(idx % CPR);
  const long long row = min(idx / CPR, n_rows - 1);      // token * n_heads + head (whole groups stay together)
  const bool live = idx / CPR < n_rows;
  const int head = (int)(row % n_heads);
  const long long tok = row / n_heads;
  const u32x4* src = q + row * (D / 8) + chunk * 2;
  const u32x4 lo = src[0], hi = src[1];
  float m = amax16(lo, hi, pre);
#pragma unroll
  for (int o = CPR / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, CPR));
  const int e = tile_exponent(m);
  if (!live) return;
  if (chunk == 0) q_exp[(long long)head * total + tok] = (unsigned char)(127 - e);
  q8[((long long)head * total + tok) * CPR + chunk] = quantize16(lo, hi, pre, pow2f(e));
}

// One workgroup packs one (unit, head): 64 keys of k into the swizzled K unit and the same 64
// rows of v, transposed and key-permuted, into the V^T unit, each with the unit's own scale.
template <int D>
__global__ __launch_bounds__(256) void fp8_pack_kv_kernel(const u32x4* __restrict__ k,
                                                          const u32x4* __restrict__ v,
                                                          u32x4* __restrict__ k8, u32x4* __restrict__ vT8,
                                                          uint32_t* __restrict__ unit_scale,
                                                          const Fp8ClipTable clips, int unit_base, int n_units,
                                                          int n_heads) {
  constexpr int CPR = D / 16;
  constexpr int PER = kF8Unit * CPR / 256;     // chunks per thread and tensor
  __shared__ __attribute__((aligned(16))) unsigned char vb[kF8Unit][D + 16];   // padded rows
  __shared__ float red[2][4];
  const int unit = unit_base + blockIdx.x, head = blockIdx.y;   // the units of this run's clips
  int lo = 0, hi = clips.n;               // last clip whose first unit is <= unit (skips empty clips)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (clips.unit0[mid] <= unit) lo = mid; else hi = mid;
  }
  const int key0 = clips.cu[lo] + (unit - clips.unit0[lo]) * kF8Unit;
  const int valid = min(kF8Unit, clips.cu[lo + 1] - key0);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  // pass 1: the raw rows into registers, the unit's largest magnitudes
  u32x4 kraw[PER][2], vraw[PER][2];
  float mk = 0.f, mv = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int oc = threadIdx.x + 256 * i;
    const int r = oc / CPR, pc = oc % CPR;
    const int lc = pc ^ k_swz<D>(r);
    kraw[i][0] = kraw[i][1] = vraw[i][0] = vraw[i][1] = zero;
    if (r < valid) {
      const size_t src = ((size_t)(key0 + r) * n_heads + head) * (D / 8) + lc * 2;
      kraw[i][0] = k[src]; kraw[i][1] = k[src + 1];
      const size_t srcv = ((size_t)(key0 + r) * n_heads + head) * (D / 8) + pc * 2;
      vraw[i][0] = v[srcv]; vraw[i][1] = v[srcv + 1];
    }
    mk = fmaxf(mk, amax16(kraw[i][0], kraw[i][1], 1.0f));
    mv = fmaxf(mv, amax16(vraw[i][0], vraw[i][1], 1.0f));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { mk = fmaxf(mk, __shfl_xor(mk, o, 64)); mv = fmaxf(mv, __shfl_xor(mv, o, 64)); }
  if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = mk; red[1][threadIdx.x >> 6] = mv; }
  __syncthreads();
  const int ek = tile_exponent(fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3])));
  const int ev = tile_exponent(fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3])));
  if (threadIdx.x == 0)
    unit_scale[(size_t)head * n_units + unit] = (uint32_t)(127 - ek) | ((uint32_t)(127 - ev) << 8) | 0x7f7f0000u;
  // pass 2: quantise with the unit's scales
  const float sk = pow2f(ek), sv = pow2f(ev);
  u32x4* kdst = k8 + ((size_t)head * n_units + unit) * (kF8Unit * CPR);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int oc = threadIdx.x + 256 * i;
    const int r = oc / CPR, pc = oc % CPR;
    kdst[oc] = quantize16(kraw[i][0], kraw[i][1], 1.0f, sk);           // (zero rows stay zero)
    *reinterpret_cast<u32x4*>(&vb[r][pc * 16]) = quantize16(vraw[i][0], vraw[i][1], 1.0f, sv);   // vb[key][d]
  }
  __syncthreads();
  u32x4* vdst = vT8 + ((size_t)head * n_units + unit) * (D * 4);
  for (int oc = threadIdx.x; oc < D * 4; oc += 256) {
    const int d = oc >> 2, pc = oc & 3;
    const int lc = pc ^ v_swz(d);
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int b = lc * 16 + i;              // logical byte of the row: lane group g, slot j
      const int g = b >> 5, j = b & 31;
      const int key = 32 * (j >> 4) + 8 * ((j & 15) >> 2) + 4 * g + (j & 3);
      const uint32_t byte = vb[key][d];
      w[i >> 2] = (i & 3) == 0 ? byte : (w[i >> 2] | (byte << (8 * (i & 3))));
    }
    const u32x4 o = {w[0], w[1], w[2], w[3]};
    vdst[oc] = o;
  }
}

// ---------------------------------------------------------------- forward
template <int D>
__global__ __launch_bounds__(kF8Waves * 64, 2)
void attn_fwd_fp8_kernel(const unsigned char* __restrict__ q8, const unsigned char* __restrict__ k8,
                         const unsigned char* __restrict__ vT8, __bf16* __restrict__ out,
                         const unsigned char* __restrict__ q_exp, const uint32_t* __restrict__ unit_scale,
                         float* __restrict__ lse, const Fp8SegTable segs, const UnitMap um, const TileIndex ti,
                         int total, int n_heads, int n_units) {
  constexpr int KS = D / 64;            // instructions per 32-key score tile
  constexpr int DB = D / 32;            // 32-row blocks of O^T
  constexpr int UB = kF8Unit * D;       // bytes of a K unit and of a V^T unit
  constexpr int kLoadWaves = UB / 1024; // waves that take part in staging a unit (1 KB each)

  extern __shared__ __attribute__((aligned(16))) char smem[];   // ring of (K unit, V^T unit), then the units' scale words
  constexpr int kScaleBase = kF8Ring * 2 * UB;                  // one 16-byte cell per ring slot

  int head, tile;
  if (!map_unit(um, blockIdx.x, head, tile)) return;
  int seq, tq;
  locate_tile(ti, segs.n, tile, seq, tq);
  const int seg_a = segs.start[seq], seg_b = seg_a + segs.len[seq];
  const int q0 = seg_a + tq * kF8Rows;
  const int unit0 = segs.unit0[seq];
  const int n_u = (segs.len[seq] + kF8Unit - 1) / kF8Unit;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane & 31, g = lane >> 5;

  // ---- Q operand: row of this lane's query, bytes ks*64 + 32g .. +31
  const int qrow = q0 + wave * 32 + c;
  i32x8 qreg[KS];
  {
    const unsigned char* qp = q8 + ((size_t)head * total + min(qrow, seg_b - 1)) * D + 32 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const u32x4 lo = *reinterpret_cast<const u32x4*>(qp + ks * 64);
      const u32x4 hi = *reinterpret_cast<const u32x4*>(qp + ks * 64 + 16);
      qreg[ks] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
    }
  }
  // block scale of this lane's query row (byte 0 of the register is the one the instruction reads)
  const int q_scale = (int)q_exp[(size_t)head * total + min(qrow, seg_b - 1)];

  // ---- staging: a unit is UB contiguous bytes in each packed buffer; wave w copies bytes
  // [w*1024, w*1024 + 1024) of it, lane L its 16-byte chunk L.  Units past the clip's last one
  // re-request the last unit (never used) so every wave keeps the same number of loads in flight.
  const unsigned char* kbase = k8 + (size_t)head * n_units * UB;
  const unsigned char* vbase = vT8 + (size_t)head * n_units * UB;
  const uint32_t lane_off = (uint32_t)(wave * 1024 + lane * 16);
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(smem) + wave * 1024);
  const uint32_t scale_lds = __builtin_amdgcn_readfirstlane(lds_addr_of(smem) + kScaleBase);
  const uint32_t* sbase = unit_scale + (size_t)head * n_units;
  auto issue_unit = [&](int u, int slot) {
    // the unit's scale word first (one lane of the workgroup), so that in every wavefront the two
    // youngest loads in flight are the unit's tiles and wait_vmcnt<2> keeps its meaning
    if (tid == 0) lds_dma4(sbase, (uint32_t)(unit0 + min(u, n_u - 1)) * 4u, scale_lds + slot * 16);
    if (wave < kLoadWaves) {
      const uint32_t off = (uint32_t)(unit0 + min(u, n_u - 1)) * UB + lane_off;
      lds_dma16(kbase, off, wave_lds + slot * 2 * UB);
      lds_dma16(vbase, off, wave_lds + slot * 2 * UB + UB);
    }
  };

  // ---- per-lane LDS offsets
  // K tile t, step ks: row 32t + c, logical chunks ks*4 + 2g and +1
  int koff[2][KS][2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int r = 32 * t + c;
        koff[t][ks][h] = r * D + (((ks * 4 + 2 * g + h) ^ k_swz<D>(r)) << 4);
      }
  // V^T block db: row db*32 + c, logical chunks 2g and 2g+1
  int voff[DB][2];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int d = db * 32 + c;
      voff[db][h] = d * 64 + (((2 * g + h) ^ v_swz(d)) << 4);
    }

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) oacc[db] = zero16;
  // The packed q carries scale * log2(e) and the instruction undoes the tiles' scales, so the score
  // instruction's result is the exponent in log2 units; its accumulator starts at minus the reference point, so the
  // exponential needs no multiply-subtract at all.
  f32x16 minit = zero16;              // -m_ref in every register
  float m_ref = 0.f, l_run = 0.f;     // reference point (log2 units, shifted) and running sum of scaled P

  issue_unit(0, 0);
  issue_unit(1, 1);

  // ---- the three stages of a unit
  f32x16 s[2];     // S^T(u) - m_ref for the unit's two 32-key tiles
  i32x8 pb;        // P(u), scaled by 2^6, as E4M3
  int us_prev = kScaleOne;   // scale word of the unit whose P V product comes next
  auto scores = [&](const char* kt, int u, int us) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)   // k unit scale (byte 0 of us) x q row scale
        s[t] = mfma_f8<0, 0>(lds_read_32b(kt, koff[t][ks][0], koff[t][ks][1]), qreg[ks], ks == 0 ? minit : s[t], us,
                             q_scale);
    const int j0 = seg_a + u * kF8Unit;
    if (j0 + kF8Unit > seg_b) {       // keys past the clip end (last unit only)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (j0 + 32 * t + 8 * (r >> 2) + 4 * g + (r & 3) >= seg_b) s[t][r] = -INFINITY;
    }
  };
  auto softmax = [&](int u) {
    // scaled exponentials against the current reference (s already holds score - m_ref)
    float p[2][16];
    float lsum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[t][r] = fast_exp2(s[t][r]);
        lsum += p[t][r];
      }
    // every scaled P <= lsum, so lsum <= 448 keeps all of them finite in E4M3 (overflow fails too).
    // Unit 0 always takes this path: it sets the first reference point from its exact row max.
    if (u == 0 || __builtin_amdgcn_ballot_w64(!(lsum <= kF8SafeSum)) != 0) {
      // move the reference to the running max (minus the 2^6 headroom), redo the unit, rescale sums and O
      float mx = s[0][0];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
      float delta = pair_max(mx) - kF8PShift;          // how far the reference has to move
      if (u != 0) delta = fmaxf(delta, 0.f);           // it only ever moves up
      const float alpha = fast_exp2(-delta);
      m_ref += delta;
#pragma unroll
      for (int r = 0; r < 16; ++r) minit[r] = -m_ref;
      lsum = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[t][r] = fast_exp2(s[t][r] - delta);
          lsum += p[t][r];
        }
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    l_run += lsum;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int w = 0; w < 4; ++w)
        pb[4 * t + w] = (int)pack_fp8x4(p[t][4 * w], p[t][4 * w + 1], p[t][4 * w + 2], p[t][4 * w + 3]);
  };
  auto accumulate = [&](const char* vt, int us) {   // O^T += 2^-e_v V^T P^T  (v unit scale: byte 1 of us)
    i32x8 va[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) va[db] = lds_read_32b(vt, voff[db][0], voff[db][1]);
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[db] = mfma_f8<1, 0>(va[db], pb, oacc[db], us, kScaleOne);
  };

  // ---- the unit loop.  A workgroup barrier per unit keeps the two wavefronts of a SIMD in step,
  // so if both ran the stages in the same order they would want the matrix pipe at the same
  // time and the VALU at the same time (measured: the two add up).  Instead waves 0-3
  // ("leaders") and 4-7 ("followers", the other wave of each SIMD) run them in opposite phase
  // between two barriers:
  //     leader  :  PV(u-1), S(u)   [matrix pipe]   then   softmax(u)       [VALU]
  //     follower:  softmax(u-1)    [VALU]          then   PV(u-1), S(u)    [matrix pipe]
  // Both read K(u) and V(u-1) in interval u; the loads issued there bring unit u+2 into the
  // slot of unit u-2 (ring of four).  SLOT = u % 4 is a compile-time constant so that every
  // LDS offset is an immediate.
  static_assert(kF8Ring == 4, "the unit loop is unrolled over the ring");
  auto interval = [&](auto slot_c, auto lead_c, auto first_c, int u) {
    constexpr int SLOT = decltype(slot_c)::value;
    constexpr bool LEAD = decltype(lead_c)::value != 0;
    constexpr bool FIRST = decltype(first_c)::value != 0;
    wait_vmcnt<2>();          // unit u has landed (unit u+1 may still be in flight) ...
    __syncthreads();          // ... for every wave, and every wave is done with unit u-2
    issue_unit(u + 2, (SLOT + 2) % kF8Ring);
    const char* kt = smem + SLOT * 2 * UB;
    const char* vt_prev = smem + ((SLOT + kF8Ring - 1) % kF8Ring) * 2 * UB + UB;
    const int us = *reinterpret_cast<const int*>(smem + kScaleBase + SLOT * 16);   // unit u's scale word
    // (a wave in its matrix phase takes the issue slot before the SIMD's other wave, which
    // is in its VALU phase then: measured 1.3% over equal priorities)
    if constexpr (LEAD) {
      __builtin_amdgcn_s_setprio(1);
      if constexpr (!FIRST) accumulate(vt_prev, us_prev);
      scores(kt, u, us);
      __builtin_amdgcn_s_setprio(0);
      softmax(u);
    } else {
      if constexpr (!FIRST) softmax(u - 1);
      __builtin_amdgcn_s_setprio(1);
      if constexpr (!FIRST) accumulate(vt_prev, us_prev);
      scores(kt, u, us);
      __builtin_amdgcn_s_setprio(0);
    }
    us_prev = us;
  };
  auto run = [&](auto lead_c) {
    interval(IntC<0>{}, lead_c, IntC<1>{}, 0);
    for (int u = 1; u < n_u; u += 4) {
      interval(IntC<1>{}, lead_c, IntC<0>{}, u);
      if (u + 1 < n_u) interval(IntC<2>{}, lead_c, IntC<0>{}, u + 1);
      if (u + 2 < n_u) interval(IntC<3>{}, lead_c, IntC<0>{}, u + 2);
      if (u + 3 < n_u) interval(IntC<0>{}, lead_c, IntC<0>{}, u + 3);
    }
    // drain: the last unit's remaining stages (its V unit is still in its slot)
    if constexpr (decltype(lead_c)::value == 0) softmax(n_u - 1);
    accumulate(smem + ((n_u - 1) % kF8Ring) * 2 * UB + UB, us_prev);
  };
  if (wave < kF8Waves / 2) run(IntC<1>{}); else run(IntC<0>{});
  wait_vmcnt<0>();   // no load may still be writing LDS when the workgroup ends

  // ---- epilogue: out = O / l (the v scales were applied by the matrix instruction), lse in natural-log units
  const float l_tot = pair_sum(l_run);
  const float inv = 1.0f / l_tot;
  if (qrow < seg_b && g == 0) lse[(size_t)head * total + qrow] = (m_ref + __log2f(l_tot)) * kF8Ln2;
  __syncthreads();   // the ring is free: each wavefront turns its tile through a piece of it
  const int row0 = q0 + wave * 32;
  store_tile_rows<D>(smem + wave * (32 * D * 2), oacc, inv, out + ((size_t)row0 * n_heads + head) * D,
                     (size_t)n_heads * D, seg_b - row0);
}

// ---------------------------------------------------------------- launchers
// scales buffer: q row exponents (n_heads * total bytes, padded to 256), then the units' scale words
static size_t unit_scale_offset(int total, int n_heads) { return ((size_t)total * n_heads + 255) / 256 * 256; }

template <int D>
static hipError_t pack_q_d(const void* q, int total, int n_heads, float pre, void* q8, void* scales,
                           hipStream_t stream) {
  const long long chunks = (long long)total * n_heads * (D / 16);
  return launch(fp8_pack_q_kernel<D>, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, stream,
                (const u32x4*)q, (u32x4*)q8, (unsigned char*)scales, pre, total, n_heads);
}

hipError_t launch_fp8_pack_q(const void* q, int total, int n_heads, int head_dim, float pre, void* q8,
                             void* scales, hipStream_t stream) {
  if (total == 0) return hipSuccess;
  if (head_dim == 128) return pack_q_d<128>(q, total, n_heads, pre, q8, scales, stream);
  return pack_q_d<64>(q, total, n_heads, pre, q8, scales, stream);
}

// k, v of one run of clips: units [clips.unit0[0], clips.unit0[clips.n]) of the call's n_units
hipError_t launch_fp8_pack_kv(const void* k, const void* v, const Fp8ClipTable& clips, int n_units, int total,
                              int n_heads, int head_dim, void* k8, void* vT8, void* scales, hipStream_t stream) {
  const int unit_base = clips.unit0[0], run_units = clips.unit0[clips.n] - unit_base;
  if (run_units == 0) return hipSuccess;
  uint32_t* us = reinterpret_cast<uint32_t*>(static_cast<char*>(scales) + unit_scale_offset(total, n_heads));
  if (head_dim == 128)
    return launch(fp8_pack_kv_kernel<128>, dim3(run_units, n_heads), dim3(256), 0, stream, (const u32x4*)k,
                  (const u32x4*)v, (u32x4*)k8, (u32x4*)vT8, us, clips, unit_base, n_units, n_heads);
  return launch(fp8_pack_kv_kernel<64>, dim3(run_units, n_heads), dim3(256), 0, stream, (const u32x4*)k,
                (const u32x4*)v, (u32x4*)k8, (u32x4*)vT8, us, clips, unit_base, n_units, n_heads);
}

template <int D>
static hipError_t fwd_fp8_d(const void* q8, const void* k8, const void* vT8, const void* scales,
                            const Fp8SegTable& segs, int n_units, int total, int n_heads,
                            void* out, float* lse, hipStream_t stream) {
  const TileIndex ti = make_tile_index<false>(segs, kF8Rows);
  const int tiles = count_tiles(ti);
  if (tiles == 0) return hipSuccess;
  UnitMap um = make_unit_map(tiles, n_heads);
  constexpr int lds = kF8Ring * 2 * kF8Unit * D + kF8Ring * 16;
  auto kern = attn_fwd_fp8_kernel<D>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  const unsigned char* q_exp = static_cast<const unsigned char*>(scales);
  const uint32_t* us = reinterpret_cast<const uint32_t*>(q_exp + unit_scale_offset(total, n_heads));
  return launch(kern, dim3(um.chunk * kNumXcd), dim3(kF8Waves * 64), lds, stream, (const unsigned char*)q8,
                (const unsigned char*)k8, (const unsigned char*)vT8, (__bf16*)out, q_exp, us, lse, segs, um, ti, total,
                n_heads, n_units);
}

hipError_t launch_attn_fwd_fp8(const void* q8, const void* k8, const void* vT8, const void* scales,
                               const Fp8SegTable& segs, int n_units, int total, int n_heads, int head_dim,
                               void* out, float* lse, hipStream_t stream) {
  if (head_dim == 128)
    return fwd_fp8_d<128>(q8, k8, vT8, scales, segs, n_units, total, n_heads, out, lse, stream);
  return fwd_fp8_d<64>(q8, k8, vT8, scales, segs, n_units, total, n_heads, out, lse, stream);
}

size_t fp8_scales_bytes(int total, int n_heads, int n_units) {
  return unit_scale_offset(total, n_heads) + (size_t)n_units * n_heads * 4;
}

}  // namespace vfm
