// C ABI of libvfm: argument validation, clip tables, launches.  No allocation, no sync.
#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <mutex>

#include "vfm_common.h"

namespace {

using vfm::RopeTable;
using vfm::SegTable;
using vfm::XSegTable;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// max_seqs < 0: any number of clips (the call is cut into runs, see below)
int check_shape(int n_seqs, int total_tokens, int n_heads, int head_dim, int max_seqs = -1) {
  if (n_seqs < 0 || (max_seqs >= 0 && n_seqs > max_seqs) || total_tokens < 0 || n_heads < 1 || n_heads > 65535)
    return VFM_ERR_SHAPE;
  if (head_dim != 64 && head_dim != 128) return VFM_ERR_SHAPE;
  // the direct-to-LDS loads address a tensor with 32-bit byte offsets
  if ((long long)total_tokens * n_heads * head_dim * 2 > 0xffffffffLL) return VFM_ERR_SHAPE;
  return VFM_OK;
}

int check_cu(const int32_t* cu, int n_seqs, int total_tokens) {
  if (cu[0] != 0) return VFM_ERR_CU_SEQLENS;
  for (int s = 0; s < n_seqs; ++s)
    if (cu[s + 1] < cu[s]) return VFM_ERR_CU_SEQLENS;
  if (cu[n_seqs] != total_tokens) return VFM_ERR_CU_SEQLENS;
  return VFM_OK;
}

// Runs.  The clip tables travel to the kernels by value, in kernel-argument memory, and hold
// VFM_MAX_SEQS clips (VFM_MAX_XSEQS cross-attention sequences).  A call with more clips is cut
// into consecutive launches on the caller's stream over runs of at most that many clips in
// packed order: clips are independent of each other, a run's tokens are one contiguous
// range, and every output row belongs to exactly one run.  The builders below therefore take
// a pointer to the run's first boundary (values stay absolute packed positions) and the
// run's number of clips.

// Non-empty clips, longest first (ties keep packed order): the tile scheduler
// hands out the most expensive tiles first.
void build_seg_table(const int32_t* cu, int n_seqs, SegTable* t) {
  int order[VFM_MAX_SEQS];
  int n = 0;
  for (int s = 0; s < n_seqs; ++s)
    if (cu[s + 1] > cu[s]) order[n++] = s;
  std::stable_sort(order, order + n, [&](int a, int b) {
    return (cu[a + 1] - cu[a]) > (cu[b + 1] - cu[b]);
  });
  t->n = n;
  for (int i = 0; i < n; ++i) {
    t->start[i] = cu[order[i]];
    t->len[i] = cu[order[i] + 1] - cu[order[i]];
  }
  for (int i = n; i < VFM_MAX_SEQS; ++i) { t->start[i] = 0; t->len[i] = 0; }
}

// Cross-attention: a sequence with queries needs at least one key (checked over the whole call
// before anything is launched).
int check_xseqs(const int32_t* cu_q, const int32_t* cu_kv, int n_seqs) {
  for (int s = 0; s < n_seqs; ++s)
    if (cu_q[s + 1] > cu_q[s] && cu_kv[s + 1] == cu_kv[s]) return VFM_ERR_CU_SEQLENS;
  return VFM_OK;
}

// Cross-attention sequences of one run, most (query x key) pairs first.  Sequences with neither
// queries nor keys are dropped.
void build_xseg_table(const int32_t* cu_q, const int32_t* cu_kv, int n_seqs, XSegTable* t) {
  int order[VFM_MAX_XSEQS];
  int n = 0;
  for (int s = 0; s < n_seqs; ++s)
    if (cu_q[s + 1] > cu_q[s] || cu_kv[s + 1] > cu_kv[s]) order[n++] = s;
  auto pairs = [&](int s) { return (long long)(cu_q[s + 1] - cu_q[s]) * (cu_kv[s + 1] - cu_kv[s]); };
  std::stable_sort(order, order + n, [&](int a, int b) { return pairs(a) > pairs(b); });
  t->n = n;
  for (int i = 0; i < VFM_MAX_XSEQS; ++i) {
    const bool live = i < n;
    t->qs[i] = live ? cu_q[order[i]] : 0;
    t->ql[i] = live ? cu_q[order[i] + 1] - cu_q[order[i]] : 0;
    t->ks[i] = live ? cu_kv[order[i]] : 0;
    t->kl[i] = live ? cu_kv[order[i] + 1] - cu_kv[order[i]] : 0;
  }
}

// Per-clip grids must match the clip lengths (an empty clip may have any grid with a zero
// extent); max_frames > 0 also bounds T (temporal attention).
int check_grids(const int32_t* thw, const int32_t* cu, int n_seqs, int max_frames) {
  for (int s = 0; s < n_seqs; ++s) {
    const long long T = thw[3 * s], H = thw[3 * s + 1], W = thw[3 * s + 2];
    const int len = cu[s + 1] - cu[s];
    if (len == 0 && T * H * W == 0 && T >= 0 && H >= 0 && W >= 0) continue;
    if (T <= 0 || H <= 0 || W <= 0 || T * H * W != len) return VFM_ERR_THW;
    if (max_frames > 0 && T > max_frames) return VFM_ERR_THW;
  }
  return VFM_OK;
}

// Temporal attention, one run of (validated) clips: packed token offsets and pixel offsets
// counted from the run's first clip.
void build_temporal_table(const int32_t* thw, const int32_t* cu, int n_seqs, vfm::TemporalTable* t) {
  t->n = n_seqs;
  int pix = 0;
  for (int s = 0; s < n_seqs; ++s) {
    const int len = cu[s + 1] - cu[s];
    t->cu[s] = cu[s];
    t->pix_cu[s] = pix;
    t->hw[s] = len == 0 ? 1 : thw[3 * s + 1] * thw[3 * s + 2];
    if (len) pix += t->hw[s];
  }
  for (int s = n_seqs; s <= VFM_MAX_SEQS; ++s) {
    t->cu[s] = cu[n_seqs];
    t->pix_cu[s] = pix;
    if (s < VFM_MAX_SEQS) t->hw[s] = 1;
  }
}

constexpr int kFp8Unit = 64;   // keys per packed unit of the FP8 path

// Units of 64 keys per clip (never straddling clips), over the whole call.
size_t count_fp8_units(const int32_t* cu, int n_seqs) {
  size_t units = 0;
  for (int s = 0; s < n_seqs; ++s) units += (size_t)(cu[s + 1] - cu[s] + kFp8Unit - 1) / kFp8Unit;
  return units;
}

// Tables of one run of clips; unit_base = units of the clips before the run.  Returns the units
// of the clips before the next run.
int build_fp8_tables(const int32_t* cu, int n_seqs, int unit_base, vfm::Fp8ClipTable* clips,
                     vfm::Fp8SegTable* segs) {
  int units = unit_base;
  int unit0[VFM_MAX_SEQS];
  clips->n = n_seqs;
  for (int s = 0; s < n_seqs; ++s) {
    clips->cu[s] = cu[s];
    clips->unit0[s] = unit0[s] = units;
    units += (cu[s + 1] - cu[s] + kFp8Unit - 1) / kFp8Unit;
  }
  for (int s = n_seqs; s <= VFM_MAX_SEQS; ++s) { clips->cu[s] = cu[n_seqs]; clips->unit0[s] = units; }
  if (segs) {   // the forward kernel's schedule: non-empty clips, longest first
    int order[VFM_MAX_SEQS];
    int n = 0;
    for (int s = 0; s < n_seqs; ++s)
      if (cu[s + 1] > cu[s]) order[n++] = s;
    std::stable_sort(order, order + n, [&](int a, int b) { return (cu[a + 1] - cu[a]) > (cu[b + 1] - cu[b]); });
    segs->n = n;
    for (int i = 0; i < vfm::kFp8MaxSeqs; ++i) {
      const bool live = i < n;
      segs->start[i] = live ? cu[order[i]] : 0;
      segs->len[i] = live ? cu[order[i] + 1] - cu[order[i]] : 0;
      segs->unit0[i] = live ? unit0[order[i]] : 0;
    }
  }
  return units;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Shared by the RoPE entry points: sizes, split, theta, cu_seqlens and the per-clip grids.
int check_rope_args(const int32_t* thw, const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                    int n_heads, int head_dim, int dim_t, int dim_h, int dim_w, float theta,
                    vfm_dtype dt) {
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  if (!(theta > 0.f) || !isfinite(theta)) return VFM_ERR_SHAPE;
  if (dim_t < 0 || dim_h < 0 || dim_w < 0 || (dim_t | dim_h | dim_w) & 1 ||
      dim_t + dim_h + dim_w != head_dim)
    return VFM_ERR_SPLIT;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (st) return st;
  return check_grids(thw, cu_seqlens, n_seqs, 0);
}

// The clip table the RoPE kernels take by value, for one run of (validated) clips.
void build_rope_table(const int32_t* thw, const int32_t* cu, int n_seqs, RopeTable* tab) {
  tab->n = n_seqs;
  for (int s = 0; s < n_seqs; ++s) {
    const bool empty = cu[s + 1] == cu[s];
    tab->cu[s] = cu[s];
    tab->hw[s] = empty ? 1 : thw[3 * s + 1] * thw[3 * s + 2];
    tab->w[s] = empty ? 1 : thw[3 * s + 2];
  }
  tab->cu[n_seqs] = cu[n_seqs];
  for (int s = n_seqs; s < VFM_MAX_SEQS; ++s) { tab->cu[s + 1] = cu[n_seqs]; tab->hw[s] = 1; tab->w[s] = 1; }
}

// The HIP error behind this thread's most recent VFM_ERR_LAUNCH.
thread_local hipError_t g_last_hip_error = hipSuccess;

// Launches go through hipLaunchKernel, which returns each launch's own status: the thread's
// pending error state (which may hold another library's leftover) is neither read nor cleared.
inline int launch_status(hipError_t e) {
  if (e == hipSuccess) return VFM_OK;
  g_last_hip_error = e;
  return VFM_ERR_LAUNCH;
}

// ---- built-in scratch of the entry point that allocates nothing ---------------------------
// vfm_attn_bwd_noalloc keeps the backward's statistics (Delta, lse in log2 units, sentinels)
// here instead of in a caller workspace.  Every GPU the library runs on holds its own copy
// of the array at its own address until the process ends.  `scratch` itself is only a
// host-side handle: host code never passes it anywhere, it asks the runtime once per device
// for the device address and uses that.
constexpr size_t kNoallocRows = VFM_NOALLOC_MAX_ROWS;                  // n_heads * total_tokens
constexpr size_t kNoallocPart = kNoallocRows * sizeof(float);         // one statistics array
constexpr size_t kNoallocBytes = 2 * kNoallocPart + 256;
static __device__ __align__(256) unsigned char scratch[kNoallocBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up on the first call on
// that device, then cached).
hipError_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return hipErrorInvalidSymbol;
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return hipSuccess;
}

}  // namespace

extern "C" {

const char* vfm_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

const char* vfm_strerror(int status) {
  switch (status) {
    case VFM_OK: return "ok";
    case VFM_ERR_NULL: return "a required pointer is NULL";
    case VFM_ERR_SHAPE: return "total_tokens, n_heads, head_dim (64 or 128), a tensor beyond 4 GiB, scale or theta (> 0, finite) or eps (>= 0) out of range, or dx aliases x";
    case VFM_ERR_CU_SEQLENS: return "cu_seqlens must start at 0, be non-decreasing and end at total_tokens";
    case VFM_ERR_THW: return "each clip needs positive T, H, W with T*H*W equal to its length";
    case VFM_ERR_SPLIT: return "dim_t + dim_h + dim_w must equal head_dim, each part even and >= 0";
    case VFM_ERR_DTYPE: return "unsupported element type (only bf16)";
    case VFM_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or smaller than vfm_attn_bwd_workspace_size()";
    case VFM_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case VFM_ERR_ALIGN: return "tensor pointers must be 16-byte aligned";
    case VFM_ERR_SCRATCH: return "n_heads * total_tokens exceeds VFM_NOALLOC_MAX_ROWS, the capacity of the built-in scratch of vfm_attn_bwd_noalloc (use vfm_attn_bwd with a workspace)";
    default: return "unknown status";
  }
}

int vfm_rope3d(void* x, const int32_t* thw, const int32_t* cu_seqlens, int n_seqs,
               int total_tokens, int n_heads, int head_dim, int dim_t, int dim_h, int dim_w,
               float theta, int inverse, vfm_dtype dt, void* hip_stream) {
  if (!x || !thw || !cu_seqlens) return VFM_ERR_NULL;
  int st = check_rope_args(thw, cu_seqlens, n_seqs, total_tokens, n_heads, head_dim, dim_t, dim_h,
                           dim_w, theta, dt);
  if (st) return st;
  if (!aligned16(x)) return VFM_ERR_ALIGN;
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_SEQS) {
    RopeTable tab;
    build_rope_table(thw + 3 * s0, cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &tab);
    hipError_t e = vfm::launch_rope3d(x, tab, n_heads, head_dim, dim_t, dim_h, dim_w, theta, inverse,
                                      static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_qknorm_rope3d(const void* x, const float* gain, float eps, void* y, const int32_t* thw,
                      const int32_t* cu_seqlens, int n_seqs, int total_tokens, int n_heads,
                      int head_dim, int dim_t, int dim_h, int dim_w, float theta, vfm_dtype dt,
                      void* hip_stream) {
  if (!x || !gain || !y || !thw || !cu_seqlens) return VFM_ERR_NULL;
  int st = check_rope_args(thw, cu_seqlens, n_seqs, total_tokens, n_heads, head_dim, dim_t, dim_h,
                           dim_w, theta, dt);
  if (st) return st;
  if (!(eps >= 0.f) || !isfinite(eps)) return VFM_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(y) || (reinterpret_cast<uintptr_t>(gain) & 3u)) return VFM_ERR_ALIGN;
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_SEQS) {
    RopeTable tab;
    build_rope_table(thw + 3 * s0, cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &tab);
    hipError_t e = vfm::launch_qknorm_rope3d(x, y, gain, eps, tab, n_heads, head_dim, dim_t, dim_h, dim_w,
                                             theta, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_qknorm_rope3d_bwd(const void* x, const float* gain, float eps, const void* dy, void* dx,
                          float* dgain, const int32_t* thw, const int32_t* cu_seqlens, int n_seqs,
                          int total_tokens, int n_heads, int head_dim, int dim_t, int dim_h,
                          int dim_w, float theta, vfm_dtype dt, void* hip_stream) {
  if (!x || !gain || !dy || !dx || !dgain || !thw || !cu_seqlens) return VFM_ERR_NULL;
  int st = check_rope_args(thw, cu_seqlens, n_seqs, total_tokens, n_heads, head_dim, dim_t, dim_h,
                           dim_w, theta, dt);
  if (st) return st;
  if (!(eps >= 0.f) || !isfinite(eps)) return VFM_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) ||
      ((reinterpret_cast<uintptr_t>(gain) | reinterpret_cast<uintptr_t>(dgain)) & 3u))
    return VFM_ERR_ALIGN;
  if (dx == x) return VFM_ERR_SHAPE;   // dx may overwrite dy, never x
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = vfm::launch_zero_f32(dgain, head_dim, stream);   // every run adds its share to dgain
  if (e != hipSuccess) return launch_status(e);
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_SEQS) {
    RopeTable tab;
    build_rope_table(thw + 3 * s0, cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &tab);
    e = vfm::launch_qknorm_rope3d_bwd(x, dy, dx, gain, eps, dgain, tab, n_heads, head_dim, dim_t, dim_h,
                                      dim_w, theta, stream);
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_attn_fwd(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                 int n_seqs, int total_tokens, int n_heads, int head_dim, float scale, void* out,
                 float* lse, vfm_dtype dt, void* hip_stream) {
  if (!q || !k || !v || !cu_seqlens || !out || !lse) return VFM_ERR_NULL;
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  if (!(scale > 0.f) || !isfinite(scale)) return VFM_ERR_SHAPE;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (st) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse))
    return VFM_ERR_ALIGN;
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_SEQS) {
    SegTable segs;
    build_seg_table(cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &segs);
    hipError_t e = vfm::launch_attn_fwd(q, k, v, segs, total_tokens, n_heads, head_dim, scale, out, lse,
                                        static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_schedule_units(const int32_t* cu_seqlens, int n_seqs, int total_tokens, int n_heads,
                       int rows_per_tile, int32_t* units, int capacity, int* n_blocks) {
  if (!cu_seqlens || !n_blocks || (!units && capacity > 0)) return VFM_ERR_NULL;
  if (n_seqs < 0 || total_tokens < 0 || n_heads < 1 || n_heads > 65535 || rows_per_tile < 1 || capacity < 0)
    return VFM_ERR_SHAPE;
  if (int st = check_cu(cu_seqlens, n_seqs, total_tokens)) return st;
  // exactly what the launchers and kernels do, run after run: count the tiles, build the unit
  // map, and ask the kernels' own mapping which unit each workgroup of the grid takes
  for (int pass = 0; pass < 2; ++pass) {
    int at = 0;
    for (int s0 = 0; s0 < n_seqs || s0 == 0; s0 += VFM_MAX_SEQS) {
      SegTable segs;
      build_seg_table(cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &segs);
      const vfm::TileIndex ti = vfm::make_tile_index<false>(segs, rows_per_tile);
      const vfm::UnitMap um = vfm::make_unit_map(vfm::count_tiles(ti), n_heads);
      const int grid = um.chunk * vfm::kNumXcd;
      if (pass == 1)
        for (int b = 0; b < grid; ++b) {
          int32_t* u = units + 3 * (at + b);
          int head, tile;
          if (!vfm::map_unit(um, b, head, tile)) {
            u[0] = -1;
            u[1] = u[2] = 0;
            continue;
          }
          int s, t;
          vfm::locate_tile(ti, segs.n, tile, s, t);
          const int first = segs.q_start(s) + t * rows_per_tile;
          u[0] = head;
          u[1] = first;
          u[2] = std::min(rows_per_tile, segs.q_start(s) + segs.q_len(s) - first);
        }
      at += grid;
      if (n_seqs == 0) break;
    }
    if (pass == 0) {
      *n_blocks = at;
      if (at > capacity) return VFM_ERR_SHAPE;
    }
  }
  return VFM_OK;
}

int vfm_attn_fwd_tile_rows(const int32_t* cu_seqlens, int n_seqs, int total_tokens, int head_dim,
                           int run, int* rows_per_tile) {
  if (!cu_seqlens || !rows_per_tile) return VFM_ERR_NULL;
  const int n_runs = n_seqs <= 0 ? 1 : (n_seqs + VFM_MAX_SEQS - 1) / VFM_MAX_SEQS;
  if (n_seqs < 0 || total_tokens < 0 || (head_dim != 64 && head_dim != 128) || run < 0 || run >= n_runs)
    return VFM_ERR_SHAPE;
  if (int st = check_cu(cu_seqlens, n_seqs, total_tokens)) return st;
  SegTable segs;
  const int s0 = run * VFM_MAX_SEQS;
  build_seg_table(cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &segs);
  *rows_per_tile = vfm::fwd_tile_rows(segs, head_dim);
  return VFM_OK;
}

size_t vfm_attn_bwd_workspace_size(int total_tokens, int n_heads, int head_dim) {
  if (check_shape(0, total_tokens, n_heads, head_dim)) return 0;
  const size_t rows = (size_t)total_tokens * n_heads;
  return 2 * align_up(rows * sizeof(float), 256) + 256;   // Delta, lse in log2 units, sentinels
}

size_t vfm_xattn_bwd_workspace_size(int total_q, int total_kv, int n_heads, int head_dim) {
  const size_t stats = vfm_attn_bwd_workspace_size(total_q, n_heads, head_dim);
  if (stats == 0 || check_shape(0, total_kv, n_heads, head_dim)) return 0;
  // + fp32 dK and dV accumulators for the query-split pass
  return stats + align_up((size_t)2 * total_kv * n_heads * head_dim * sizeof(float), 256);
}

namespace {

// Both self-attention backward entry points, once their statistics buffers are known.
int attn_bwd_common(const void* q, const void* k, const void* v, const void* out, const float* lse,
                    const void* dout, const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                    int n_heads, int head_dim, float scale, void* dq, void* dk, void* dv, float* delta,
                    float* lse2, float* sentinel, hipStream_t stream) {
  hipError_t e = vfm::launch_bwd_prepare(out, dout, lse, delta, lse2, sentinel, total_tokens, n_heads,
                                         head_dim, stream);
  if (e != hipSuccess) return launch_status(e);
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_SEQS) {
    SegTable segs;
    build_seg_table(cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &segs);
    e = vfm::launch_attn_bwd(q, k, v, out, lse, dout, segs, total_tokens, n_heads, head_dim, scale, dq, dk,
                             dv, delta, lse2, sentinel, nullptr, 0, 0, 0, stream);
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int check_attn_bwd_args(const void* q, const void* k, const void* v, const void* out, const float* lse,
                        const void* dout, const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                        int n_heads, int head_dim, float scale, void* dq, void* dk, void* dv, vfm_dtype dt) {
  if (!q || !k || !v || !out || !lse || !dout || !cu_seqlens || !dq || !dk || !dv)
    return VFM_ERR_NULL;
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  if (!(scale > 0.f) || !isfinite(scale)) return VFM_ERR_SHAPE;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (st) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse) ||
      !aligned16(dout) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
    return VFM_ERR_ALIGN;
  return VFM_OK;
}

}  // namespace

int vfm_attn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                 const void* dout, const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                 int n_heads, int head_dim, float scale, void* dq, void* dk, void* dv,
                 void* workspace, size_t workspace_bytes, vfm_dtype dt, void* hip_stream) {
  int st = check_attn_bwd_args(q, k, v, out, lse, dout, cu_seqlens, n_seqs, total_tokens, n_heads, head_dim,
                               scale, dq, dk, dv, dt);
  if (st) return st;
  if (total_tokens == 0) return VFM_OK;
  const size_t need = vfm_attn_bwd_workspace_size(total_tokens, n_heads, head_dim);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
    return VFM_ERR_WORKSPACE;
  float* delta = static_cast<float*>(workspace);
  const size_t part = (need - 256) / 2;
  float* lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + part);
  float* sentinel = reinterpret_cast<float*>(static_cast<char*>(workspace) + 2 * part);
  return attn_bwd_common(q, k, v, out, lse, dout, cu_seqlens, n_seqs, total_tokens, n_heads, head_dim, scale,
                         dq, dk, dv, delta, lse2, sentinel, static_cast<hipStream_t>(hip_stream));
}

int vfm_attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* out,
                         const float* lse, const void* dout, const int32_t* cu_seqlens, int n_seqs,
                         int total_tokens, int n_heads, int head_dim, float scale, void* dq, void* dk,
                         void* dv, vfm_dtype dt, void* hip_stream) {
  int st = check_attn_bwd_args(q, k, v, out, lse, dout, cu_seqlens, n_seqs, total_tokens, n_heads, head_dim,
                               scale, dq, dk, dv, dt);
  if (st) return st;
  if ((size_t)total_tokens * (size_t)n_heads > kNoallocRows) return VFM_ERR_SCRATCH;
  if (total_tokens == 0) return VFM_OK;
  void* base = nullptr;
  hipError_t e = scratch_of_current_device(&base);
  if (e != hipSuccess) return launch_status(e);
  // the same three regions vfm_attn_bwd cuts from its workspace, at fixed places
  float* delta = static_cast<float*>(base);
  float* lse2 = reinterpret_cast<float*>(static_cast<char*>(base) + kNoallocPart);
  float* sentinel = reinterpret_cast<float*>(static_cast<char*>(base) + 2 * kNoallocPart);
  return attn_bwd_common(q, k, v, out, lse, dout, cu_seqlens, n_seqs, total_tokens, n_heads, head_dim, scale,
                         dq, dk, dv, delta, lse2, sentinel, static_cast<hipStream_t>(hip_stream));
}

int vfm_xattn_fwd(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_q,
                  const int32_t* cu_seqlens_kv, int n_seqs, int total_q, int total_kv, int n_heads,
                  int head_dim, float scale, void* out, float* lse, vfm_dtype dt, void* hip_stream) {
  if (!q || !k || !v || !cu_seqlens_q || !cu_seqlens_kv || !out || !lse) return VFM_ERR_NULL;
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_q, n_heads, head_dim);
  if (!st) st = check_shape(n_seqs, total_kv, n_heads, head_dim);
  if (st) return st;
  if (!(scale > 0.f) || !isfinite(scale)) return VFM_ERR_SHAPE;
  st = check_cu(cu_seqlens_q, n_seqs, total_q);
  if (!st) st = check_cu(cu_seqlens_kv, n_seqs, total_kv);
  if (!st) st = check_xseqs(cu_seqlens_q, cu_seqlens_kv, n_seqs);
  if (st) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse))
    return VFM_ERR_ALIGN;
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_XSEQS) {
    XSegTable segs;
    build_xseg_table(cu_seqlens_q + s0, cu_seqlens_kv + s0, std::min(VFM_MAX_XSEQS, n_seqs - s0), &segs);
    hipError_t e = vfm::launch_attn_fwd(q, k, v, segs, total_q, n_heads, head_dim, scale, out, lse,
                                        static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_xattn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                  const void* dout, const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_kv,
                  int n_seqs, int total_q, int total_kv, int n_heads, int head_dim, float scale,
                  void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                  vfm_dtype dt, void* hip_stream) {
  if (!q || !k || !v || !out || !lse || !dout || !cu_seqlens_q || !cu_seqlens_kv || !dq || !dk || !dv)
    return VFM_ERR_NULL;
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_q, n_heads, head_dim);
  if (!st) st = check_shape(n_seqs, total_kv, n_heads, head_dim);
  if (st) return st;
  if (!(scale > 0.f) || !isfinite(scale)) return VFM_ERR_SHAPE;
  st = check_cu(cu_seqlens_q, n_seqs, total_q);
  if (!st) st = check_cu(cu_seqlens_kv, n_seqs, total_kv);
  if (!st) st = check_xseqs(cu_seqlens_q, cu_seqlens_kv, n_seqs);
  if (st) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse) ||
      !aligned16(dout) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
    return VFM_ERR_ALIGN;
  if (total_kv == 0) return VFM_OK;     // then total_q is 0 too
  const size_t stats = vfm_attn_bwd_workspace_size(total_q, n_heads, head_dim);
  const size_t need = vfm_xattn_bwd_workspace_size(total_q, total_kv, n_heads, head_dim);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
    return VFM_ERR_WORKSPACE;
  float* delta = static_cast<float*>(workspace);
  const size_t part = (stats - 256) / 2;
  float* lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + part);
  float* sentinel = reinterpret_cast<float*>(static_cast<char*>(workspace) + 2 * part);
  float* dkv32 = reinterpret_cast<float*>(static_cast<char*>(workspace) + stats);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = vfm::launch_bwd_prepare(out, dout, lse, delta, lse2, sentinel, total_q, n_heads, head_dim, stream);
  if (e != hipSuccess) return launch_status(e);
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_XSEQS) {
    const int n = std::min(VFM_MAX_XSEQS, n_seqs - s0);
    XSegTable segs;
    build_xseg_table(cu_seqlens_q + s0, cu_seqlens_kv + s0, n, &segs);
    e = vfm::launch_attn_bwd(q, k, v, out, lse, dout, segs, total_q, n_heads, head_dim, scale, dq, dk, dv,
                             delta, lse2, sentinel, dkv32, total_kv, cu_seqlens_kv[s0], cu_seqlens_kv[s0 + n],
                             stream);
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_tattn_fwd(const void* q, const void* k, const void* v, const int32_t* thw,
                  const int32_t* cu_seqlens, int n_seqs, int total_tokens, int n_heads, int head_dim,
                  float scale, void* out, vfm_dtype dt, void* hip_stream) {
  if (!q || !k || !v || !thw || !cu_seqlens || !out) return VFM_ERR_NULL;
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  if (!(scale > 0.f) || !isfinite(scale)) return VFM_ERR_SHAPE;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (!st) st = check_grids(thw, cu_seqlens, n_seqs, 0);
  if (st) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return VFM_ERR_ALIGN;
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_SEQS) {
    vfm::TemporalTable tab;
    build_temporal_table(thw + 3 * s0, cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &tab);
    hipError_t e = vfm::launch_tattn_fwd(q, k, v, tab, n_heads, head_dim, scale, out,
                                         static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_tattn_bwd(const void* q, const void* k, const void* v, const void* dout, const int32_t* thw,
                  const int32_t* cu_seqlens, int n_seqs, int total_tokens, int n_heads, int head_dim,
                  float scale, void* dq, void* dk, void* dv, vfm_dtype dt, void* hip_stream) {
  if (!q || !k || !v || !dout || !thw || !cu_seqlens || !dq || !dk || !dv) return VFM_ERR_NULL;
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  if (!(scale > 0.f) || !isfinite(scale)) return VFM_ERR_SHAPE;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (!st) st = check_grids(thw, cu_seqlens, n_seqs, 0);
  if (st) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(dout) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv))
    return VFM_ERR_ALIGN;
  for (int s0 = 0; s0 < n_seqs; s0 += VFM_MAX_SEQS) {
    vfm::TemporalTable tab;
    build_temporal_table(thw + 3 * s0, cu_seqlens + s0, std::min(VFM_MAX_SEQS, n_seqs - s0), &tab);
    hipError_t e = vfm::launch_tattn_bwd(q, k, v, dout, tab, n_heads, head_dim, scale, dq, dk, dv,
                                         static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_fp8_pack_sizes(const int32_t* cu_seqlens, int n_seqs, int total_tokens, int n_heads,
                       int head_dim, size_t* q8_bytes, size_t* k8_bytes, size_t* vT8_bytes,
                       size_t* scales_bytes) {
  if (!cu_seqlens || !q8_bytes || !k8_bytes || !vT8_bytes || !scales_bytes) return VFM_ERR_NULL;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (st) return st;
  const size_t units = count_fp8_units(cu_seqlens, n_seqs);
  *q8_bytes = (size_t)total_tokens * n_heads * head_dim;
  *k8_bytes = units * n_heads * kFp8Unit * head_dim;
  *vT8_bytes = *k8_bytes;
  *scales_bytes = 0;
  if (*k8_bytes > 0xffffffffULL) return VFM_ERR_SHAPE;   // the kernels address a unit with a 32-bit byte offset
  *scales_bytes = vfm::fp8_scales_bytes(total_tokens, n_heads, (int)units);
  return VFM_OK;
}

int vfm_fp8_pack(const void* q, const void* k, const void* v, const int32_t* cu_seqlens, int n_seqs,
                 int total_tokens, int n_heads, int head_dim, float scale, void* q8, void* k8, void* vT8,
                 void* scales, vfm_dtype dt, void* hip_stream) {
  const float pre = scale * 1.4426950408889634f;   // scores come out in log2 units
  if (!q || !k || !v || !cu_seqlens || !q8 || !k8 || !vT8 || !scales) return VFM_ERR_NULL;
  if (dt != VFM_BF16) return VFM_ERR_DTYPE;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  if (!(scale > 0.f) || !isfinite(scale) || !isfinite(pre)) return VFM_ERR_SHAPE;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (st) return st;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(q8) || !aligned16(k8) || !aligned16(vT8) ||
      !aligned16(scales))
    return VFM_ERR_ALIGN;
  const size_t units = count_fp8_units(cu_seqlens, n_seqs);
  if (units * n_heads * kFp8Unit * head_dim > 0xffffffffULL) return VFM_ERR_SHAPE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = vfm::launch_fp8_pack_q(q, total_tokens, n_heads, head_dim, pre, q8, scales, stream);
  if (e != hipSuccess) return launch_status(e);
  int unit_base = 0;
  for (int s0 = 0; s0 < n_seqs; s0 += vfm::kFp8MaxSeqs) {
    vfm::Fp8ClipTable clips;
    unit_base = build_fp8_tables(cu_seqlens + s0, std::min(vfm::kFp8MaxSeqs, n_seqs - s0), unit_base, &clips, nullptr);
    e = vfm::launch_fp8_pack_kv(k, v, clips, (int)units, total_tokens, n_heads, head_dim, k8, vT8, scales, stream);
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

int vfm_attn_fwd_fp8(const void* q8, const void* k8, const void* vT8, const void* scales,
                     const int32_t* cu_seqlens, int n_seqs, int total_tokens, int n_heads, int head_dim,
                     void* out, float* lse, void* hip_stream) {
  if (!q8 || !k8 || !vT8 || !scales || !cu_seqlens || !out || !lse) return VFM_ERR_NULL;
  int st = check_shape(n_seqs, total_tokens, n_heads, head_dim);
  if (st) return st;
  st = check_cu(cu_seqlens, n_seqs, total_tokens);
  if (st) return st;
  if (!aligned16(q8) || !aligned16(k8) || !aligned16(vT8) || !aligned16(scales) || !aligned16(out) || !aligned16(lse))
    return VFM_ERR_ALIGN;
  const size_t units = count_fp8_units(cu_seqlens, n_seqs);
  if (units * n_heads * kFp8Unit * head_dim > 0xffffffffULL) return VFM_ERR_SHAPE;
  int unit_base = 0;
  for (int s0 = 0; s0 < n_seqs; s0 += vfm::kFp8MaxSeqs) {
    vfm::Fp8ClipTable clips;
    vfm::Fp8SegTable segs;
    unit_base = build_fp8_tables(cu_seqlens + s0, std::min(vfm::kFp8MaxSeqs, n_seqs - s0), unit_base, &clips, &segs);
    hipError_t e = vfm::launch_attn_fwd_fp8(q8, k8, vT8, scales, segs, (int)units, total_tokens, n_heads, head_dim,
                                            out, lse, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return launch_status(e);
  }
  return VFM_OK;
}

}  // extern "C"
