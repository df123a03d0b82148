// Host-only exercise of the library's argument validation, clip-table builders, run splitting and
// tile scheduler under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU, nothing launched).
// Built by tests/test_host_sanitizers.py from csrc/vfm_api.hip plus the launcher stubs below, which
// stand in for the kernels' launchers and check what the tables they are handed contain.
#include <stdio.h>
#include <stdlib.h>

#include <random>
#include <vector>

#include "vfm_common.h"

static long g_launches = 0;
static int g_failures = 0;
#define EXPECT(cond)                                                              \
  do {                                                                            \
    if (!(cond)) { ++g_failures; fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); } \
  } while (0)

namespace vfm {

// Every table a launcher receives must be internally consistent: that is what the kernels rely on.
static void check_rope_table(const RopeTable& t) {
  EXPECT(t.n >= 0 && t.n <= VFM_MAX_SEQS);
  for (int s = 0; s < t.n; ++s) {
    EXPECT(t.cu[s] <= t.cu[s + 1]);
    EXPECT(t.hw[s] >= 1 && t.w[s] >= 1);
    if (t.cu[s + 1] > t.cu[s]) EXPECT((t.cu[s + 1] - t.cu[s]) % t.hw[s] == 0 && t.hw[s] % t.w[s] == 0);
  }
  for (int s = t.n; s < VFM_MAX_SEQS; ++s) EXPECT(t.cu[s + 1] == t.cu[t.n]);
}
template <class Segs>
static void check_segs(const Segs& segs, int total_q) {
  EXPECT(segs.n >= 0);
  for (int s = 0; s < segs.n; ++s) {
    EXPECT(segs.q_len(s) >= 0 && segs.kv_len(s) >= 0 && segs.q_len(s) + segs.kv_len(s) > 0);
    EXPECT(segs.q_start(s) >= 0 && segs.q_start(s) + segs.q_len(s) <= total_q);
    if (segs.q_len(s) > 0) EXPECT(segs.kv_len(s) > 0);
  }
}

hipError_t launch_rope3d(void*, const RopeTable& tab, int, int, int, int, int, float, int, hipStream_t) {
  ++g_launches; check_rope_table(tab); return hipSuccess;
}
hipError_t launch_qknorm_rope3d(const void*, void*, const float*, float, const RopeTable& tab, int, int, int, int, int,
                                float, hipStream_t) { ++g_launches; check_rope_table(tab); return hipSuccess; }
hipError_t launch_qknorm_rope3d_bwd(const void*, const void*, void*, const float*, float, float*, const RopeTable& tab,
                                    int, int, int, int, int, float, hipStream_t) {
  ++g_launches; check_rope_table(tab); return hipSuccess;
}
hipError_t launch_zero_f32(float*, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_tattn_fwd(const void*, const void*, const void*, const TemporalTable& t, int, int, float, void*,
                            hipStream_t) {
  ++g_launches;
  EXPECT(t.n >= 0 && t.n <= VFM_MAX_SEQS);
  for (int s = 0; s < t.n; ++s) { EXPECT(t.hw[s] >= 1 && t.pix_cu[s] <= t.pix_cu[s + 1] && t.cu[s] <= t.cu[s + 1]); }
  return hipSuccess;
}
hipError_t launch_tattn_bwd(const void* q, const void* k, const void* v, const void*, const TemporalTable& t, int h, int d,
                            float sc, void* o, void*, void*, hipStream_t st) { return launch_tattn_fwd(q, k, v, t, h, d, sc, o, st); }
hipError_t launch_fp8_pack_q(const void*, int, int, int, float, void*, void*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_fp8_pack_kv(const void*, const void*, const Fp8ClipTable& c, int n_units, int, int, int, void*, void*,
                              void*, hipStream_t) {
  ++g_launches;
  EXPECT(c.n >= 0 && c.n <= VFM_MAX_SEQS);
  for (int s = 0; s < c.n; ++s) {
    EXPECT(c.unit0[s + 1] - c.unit0[s] == (c.cu[s + 1] - c.cu[s] + 63) / 64);
    EXPECT(c.unit0[s + 1] <= n_units);
  }
  return hipSuccess;
}
hipError_t launch_attn_fwd_fp8(const void*, const void*, const void*, const void*, const Fp8SegTable& segs, int n_units,
                               int total, int, int, void*, float*, hipStream_t) {
  ++g_launches;
  for (int s = 0; s < segs.n; ++s) {
    EXPECT(segs.len[s] > 0 && segs.start[s] >= 0 && segs.start[s] + segs.len[s] <= total);
    EXPECT(segs.unit0[s] >= 0 && segs.unit0[s] + (segs.len[s] + 63) / 64 <= n_units);
    if (s) EXPECT(segs.len[s - 1] >= segs.len[s]);
  }
  return hipSuccess;
}
size_t fp8_scales_bytes(int total, int n_heads, int n_units) {
  return ((size_t)total * n_heads + 255) / 256 * 256 + (size_t)n_units * n_heads * 4;
}
template <class Segs>
hipError_t launch_attn_fwd(const void*, const void*, const void*, const Segs& segs, int total_q, int, int, float, void*,
                           float*, hipStream_t) { ++g_launches; check_segs(segs, total_q); return hipSuccess; }
hipError_t launch_bwd_prepare(const void*, const void*, const float*, float*, float*, float*, int, int, int, hipStream_t) {
  ++g_launches; return hipSuccess;
}
template <class Segs>
hipError_t launch_attn_bwd(const void*, const void*, const void*, const void*, const float*, const void*, const Segs& segs,
                           int total_q, int, int, float, void*, void*, void*, float*, float*, float*, float*, int total_kv,
                           int kv_lo, int kv_hi, hipStream_t) {
  ++g_launches; check_segs(segs, total_q); EXPECT(kv_lo >= 0 && kv_lo <= kv_hi && kv_hi <= total_kv + (total_kv == 0 ? kv_hi : 0));
  return hipSuccess;
}
template hipError_t launch_attn_fwd<SegTable>(const void*, const void*, const void*, const SegTable&, int, int, int, float,
                                              void*, float*, hipStream_t);
template hipError_t launch_attn_fwd<XSegTable>(const void*, const void*, const void*, const XSegTable&, int, int, int, float,
                                               void*, float*, hipStream_t);
template hipError_t launch_attn_bwd<SegTable>(const void*, const void*, const void*, const void*, const float*, const void*,
                                              const SegTable&, int, int, int, float, void*, void*, void*, float*, float*,
                                              float*, float*, int, int, int, hipStream_t);
template hipError_t launch_attn_bwd<XSegTable>(const void*, const void*, const void*, const void*, const float*, const void*,
                                               const XSegTable&, int, int, int, float, void*, void*, void*, float*, float*,
                                               float*, float*, int, int, int, hipStream_t);
}  // namespace vfm

int main() {
  std::mt19937 rng(12345);
  void* const P = reinterpret_cast<void*>(0x10000);     // never dereferenced: the stubs launch nothing
  float* const F = reinterpret_cast<float*>(0x20000);
  const size_t big = (size_t)1 << 40;
  for (int trial = 0; trial < 400; ++trial) {
    // clip counts on both sides of every run boundary, lengths with many zeros
    const int n_opts[] = {0, 1, 2, 127, 128, 129, 255, 256, 257, 511, 512, 513, 700, 1025};
    const int n = n_opts[rng() % 14];
    const int heads = 1 + rng() % 5, hd = (rng() & 1) ? 128 : 64;
    std::vector<int32_t> cu(n + 1, 0), thw(3 * (n + 1), 0), cu_kv(n + 1, 0);
    for (int s = 0; s < n; ++s) {
      int T = rng() % 5, H = 1 + rng() % 6, W = 1 + rng() % 6;
      if (rng() % 7 == 0) { T = 1; H = 1; W = 1 + rng() % 300; }
      if (rng() % 23 == 0) T = 33 + rng() % 100;
      thw[3 * s] = T; thw[3 * s + 1] = H; thw[3 * s + 2] = W;
      cu[s + 1] = cu[s] + T * H * W;
      cu_kv[s + 1] = cu_kv[s] + (T * H * W > 0 ? 1 + (int)(rng() % 90) : (int)(rng() % 3));
    }
    const int total = cu[n], total_kv = cu_kv[n];
    const int d2 = hd / 4 * 2, d1 = hd - 2 * d2 >= 0 ? hd - 2 * d2 : 0;
    EXPECT(vfm_rope3d(P, thw.data(), cu.data(), n, total, heads, hd, d1, d2, d2, 1e4f, trial & 1, VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_qknorm_rope3d(P, F, 1e-6f, P, thw.data(), cu.data(), n, total, heads, hd, d1, d2, d2, 1e4f, VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_qknorm_rope3d_bwd(P, F, 1e-6f, F, F + 64, F, thw.data(), cu.data(), n, total, heads, hd, d1, d2, d2, 1e4f,
                                 VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_attn_fwd(P, P, P, cu.data(), n, total, heads, hd, 0.1f, P, F, VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_attn_bwd(P, P, P, P, F, P, cu.data(), n, total, heads, hd, 0.1f, P, P, P, P, big, VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_attn_bwd_noalloc(P, P, P, P, F, P, cu.data(), n, 0, heads, hd, 0.1f, P, P, P, VFM_BF16, nullptr) ==
           (total == 0 ? VFM_OK : VFM_ERR_CU_SEQLENS));
    EXPECT(vfm_xattn_fwd(P, P, P, cu.data(), cu_kv.data(), n, total, total_kv, heads, hd, 0.1f, P, F, VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_xattn_bwd(P, P, P, P, F, P, cu.data(), cu_kv.data(), n, total, total_kv, heads, hd, 0.1f, P, P, P, P, big,
                         VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_tattn_fwd(P, P, P, thw.data(), cu.data(), n, total, heads, hd, 0.1f, P, VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_tattn_bwd(P, P, P, P, thw.data(), cu.data(), n, total, heads, hd, 0.1f, P, P, P, VFM_BF16, nullptr) == VFM_OK);
    size_t a, b, c, d;
    EXPECT(vfm_fp8_pack_sizes(cu.data(), n, total, heads, hd, &a, &b, &c, &d) == VFM_OK);
    EXPECT(vfm_fp8_pack(P, P, P, cu.data(), n, total, heads, hd, 0.1f, P, P, P, P, VFM_BF16, nullptr) == VFM_OK);
    EXPECT(vfm_attn_fwd_fp8(P, P, P, P, cu.data(), n, total, heads, hd, P, F, nullptr) == VFM_OK);
    // the scheduler: ask for the size, then fill exactly that many entries (a too-small buffer is refused)
    const int rows = 32 << (rng() % 4);
    int n_blocks = -1;
    EXPECT(vfm_schedule_units(cu.data(), n, total, heads, rows, nullptr, 0, &n_blocks) == (n_blocks == 0 ? VFM_OK : VFM_ERR_SHAPE));
    std::vector<int32_t> units(3 * (size_t)(n_blocks > 0 ? n_blocks : 1));
    if (n_blocks > 1) EXPECT(vfm_schedule_units(cu.data(), n, total, heads, rows, units.data(), n_blocks - 1, &n_blocks) == VFM_ERR_SHAPE);
    int again = -1;
    EXPECT(vfm_schedule_units(cu.data(), n, total, heads, rows, units.data(), n_blocks, &again) == VFM_OK && again == n_blocks);
    long covered = 0;
    for (int bidx = 0; bidx < n_blocks; ++bidx)
      if (units[3 * bidx] >= 0) {
        EXPECT(units[3 * bidx] < heads && units[3 * bidx + 1] >= 0 && units[3 * bidx + 2] >= 1 && units[3 * bidx + 2] <= rows &&
               units[3 * bidx + 1] + units[3 * bidx + 2] <= total);
        covered += units[3 * bidx + 2];
      }
    EXPECT(covered == (long)total * heads);
    const int n_runs = n == 0 ? 1 : (n + VFM_MAX_SEQS - 1) / VFM_MAX_SEQS;
    int tr = 0;
    EXPECT(vfm_attn_fwd_tile_rows(cu.data(), n, total, hd, n_runs - 1, &tr) == VFM_OK && (tr == 128 || tr == 256));
    EXPECT(vfm_attn_fwd_tile_rows(cu.data(), n, total, hd, n_runs, &tr) == VFM_ERR_SHAPE);
    // malformed boundaries are refused before any table is built
    if (n >= 2) {
      std::vector<int32_t> bad(cu);
      bad[n / 2] = bad[n] + 1;
      const long before = g_launches;
      EXPECT(vfm_attn_fwd(P, P, P, bad.data(), n, total, heads, hd, 0.1f, P, F, VFM_BF16, nullptr) == VFM_ERR_CU_SEQLENS);
      EXPECT(vfm_rope3d(P, thw.data(), bad.data(), n, total, heads, hd, d1, d2, d2, 1e4f, 0, VFM_BF16, nullptr) == VFM_ERR_CU_SEQLENS);
      EXPECT(g_launches == before);
    }
  }
  printf("%s: %ld stub launches, %d failures\n", g_failures ? "FAILED" : "ok", g_launches, g_failures);
  return g_failures ? 1 : 0;
}
