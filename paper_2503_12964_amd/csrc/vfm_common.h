// Shared device helpers and launcher declarations for libvfm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "../../include/vfm.h"

namespace vfm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// MI355X: 8 XCDs, workgroups are dealt to them round-robin.  A compile-time constant on purpose: it
// is part of the device-side block -> unit mapping (the HIP runtime exposes no XCD count to ask for),
// and the library is built for this one chip.
constexpr int kNumXcd = 8;

// Non-empty clips, longest first.  Passed to kernels by value (kernel argument
// memory), so no device allocation or copy is needed for the schedule.  Self-attention:
// a clip's queries and keys are the same token range.
struct SegTable {
  int n;
  int start[VFM_MAX_SEQS];
  int len[VFM_MAX_SEQS];
  __device__ __host__ int q_start(int s) const { return start[s]; }
  __device__ __host__ int q_len(int s) const { return len[s]; }
  __device__ __host__ int kv_start(int s) const { return start[s]; }
  __device__ __host__ int kv_len(int s) const { return len[s]; }
};

// Cross-attention: sequence s owns a query range of one packed tensor and a key/value
// range of another.  Same size in kernel-argument memory as SegTable.
struct XSegTable {
  int n;
  int qs[VFM_MAX_XSEQS], ql[VFM_MAX_XSEQS], ks[VFM_MAX_XSEQS], kl[VFM_MAX_XSEQS];
  __device__ __host__ int q_start(int s) const { return qs[s]; }
  __device__ __host__ int q_len(int s) const { return ql[s]; }
  __device__ __host__ int kv_start(int s) const { return ks[s]; }
  __device__ __host__ int kv_len(int s) const { return kl[s]; }
};

// Clip table for RoPE: all clips in packed order.
struct RopeTable {
  int n;
  int cu[VFM_MAX_SEQS + 1];
  int hw[VFM_MAX_SEQS];  // H*W of the clip's latent grid
  int w[VFM_MAX_SEQS];   // W
};

// FP8 attention: keys and values are packed in units of 64 keys that never straddle a clip.
// Packed-order table for the packing pass ...
struct Fp8ClipTable {
  int n;
  int cu[VFM_MAX_SEQS + 1];     // first packed token of clip s
  int unit0[VFM_MAX_SEQS + 1];  // units of the clips before s
};
// ... and the forward kernel's schedule (non-empty clips, longest first).  The FP8 entry points
// cut a call into runs of kFp8MaxSeqs clips: with three arrays per clip and the tile index beside
// it, a 256-clip table would not fit the 4 KB of kernel arguments.
constexpr int kFp8MaxSeqs = 128;
struct Fp8SegTable {
  int n;
  int start[kFp8MaxSeqs];
  int len[kFp8MaxSeqs];
  int unit0[kFp8MaxSeqs];       // first unit of the clip in the packed buffers
  __device__ __host__ int q_start(int s) const { return start[s]; }
  __device__ __host__ int q_len(int s) const { return len[s]; }
  __device__ __host__ int kv_start(int s) const { return start[s]; }
  __device__ __host__ int kv_len(int s) const { return len[s]; }
};

// Clip table for temporal attention: packed token and pixel offsets of every clip.
struct TemporalTable {
  int n;
  int cu[VFM_MAX_SEQS + 1];      // first packed token of clip s
  int pix_cu[VFM_MAX_SEQS + 1];  // pixels (H*W) of the clips before s
  int hw[VFM_MAX_SEQS];          // H*W of clip s (1 for an empty clip)
};

// The same clips for the temporal kernels that walk sequences of more than 32 frames in
// 32-row blocks: a work unit is one block of one (pixel, head) sequence.
struct TemporalLTable {
  int n;
  int cu[VFM_MAX_SEQS + 1];      // first packed token of clip s
  int blk_cu[VFM_MAX_SEQS + 1];  // (pixel, block) pairs of the clips before s: sum of H*W * ceil(T / 32)
  int hw[VFM_MAX_SEQS];          // H*W of clip s (1 for an empty clip)
};

// Work unit u = head * tiles_per_head + tile, units split into kNumXcd
// contiguous chunks so that one XCD (one L2) walks the tiles of one head
// together.  Returns false if this workgroup has nothing to do.
struct UnitMap {
  int tiles_per_head;
  int n_units;
  int chunk;  // ceil(n_units / kNumXcd)
};

// The launch geometry of a kernel that takes one (head, tile) unit per workgroup: units are
// numbered head-major and cut into kNumXcd contiguous chunks; workgroup b belongs to XCD
// b % kNumXcd and takes unit (b % kNumXcd) * chunk + b / kNumXcd, so that the workgroups
// sharing an L2 walk neighbouring tiles of the same head.  Grid = chunk * kNumXcd.
__host__ inline UnitMap make_unit_map(int tiles_per_head, int n_heads) {
  UnitMap um;
  um.tiles_per_head = tiles_per_head;
  um.n_units = tiles_per_head * n_heads;
  um.chunk = (um.n_units + kNumXcd - 1) / kNumXcd;
  return um;
}

__host__ __device__ __forceinline__ bool map_unit(const UnitMap& um, int block, int& head, int& tile) {
  const int xcd = block % kNumXcd;
  const int local = block / kNumXcd;
  const int u = xcd * um.chunk + local;
  if (local >= um.chunk || u >= um.n_units) return false;
  head = u / um.tiles_per_head;
  tile = u - head * um.tiles_per_head;
  return true;
}

// Tiles of the sequences before s (table order) for one launch's tile height, built on the host
// and passed by value beside the sequence table.  A workgroup finds its sequence by binary
// search in it: walking the table instead costs a dependent scalar load per sequence, which with
// 256 clips in a call took as long as a short clip's whole key loop.  Tiles are cut from the
// query ranges (KV = false) or from the key/value ranges (KV = true).
struct TileIndex {
  int cu[VFM_MAX_SEQS + 1];   // cu[s] = tiles of sequences 0..s-1; entries past the table repeat the total
};

template <bool KV, class Segs>
inline TileIndex make_tile_index(const Segs& segs, int rows_per_tile) {
  TileIndex ti;
  int tiles = 0;
  for (int s = 0; s <= VFM_MAX_SEQS; ++s) {
    ti.cu[s] = tiles;
    if (s < segs.n) tiles += ((KV ? segs.kv_len(s) : segs.q_len(s)) + rows_per_tile - 1) / rows_per_tile;
  }
  return ti;
}
inline int count_tiles(const TileIndex& ti) { return ti.cu[VFM_MAX_SEQS]; }

// Tile index (over the n sequences of the table, in table order) -> sequence s and tile t within
// it: the last s with cu[s] <= tile, which skips sequences that have no tile.
__host__ __device__ __forceinline__ void locate_tile(const TileIndex& ti, int n, int tile, int& s, int& t) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (ti.cu[mid] <= tile) lo = mid; else hi = mid;
  }
  s = lo;
  t = tile - ti.cu[lo];
}

// Query rows per workgroup of the forward kernel for the sequences of one launch.  Few keys
// per sequence (cross-attention on a text prompt, packs of images): a workgroup's loop is
// short against its prologue and epilogue, so 128-row workgroups are used, two of which share
// a CU and overlap one's loads and stores with the other's loop (0.59 -> 0.55 ms for 56,320
// queries x 512 keys x 32 heads; +3-5% on packs of 256- to 484-token clips).  Each
// wavefront's arithmetic is the same.  With longer sequences the 256-row workgroup's halved
// K/V staging traffic wins.  head_dim 64 always uses 128-row workgroups.
template <class Segs>
inline int fwd_tile_rows(const Segs& segs, int head_dim) {
  if (head_dim != 128) return 128;
  int longest_kv = 0;
  for (int s = 0; s < segs.n; ++s) longest_kv = longest_kv > segs.kv_len(s) ? longest_kv : segs.kv_len(s);
  return longest_kv <= 1024 ? 128 : 256;
}

// LDS tiles hold rows of D bf16 without padding; the 16-byte chunk index within
// a row is XOR-ed with a function of the row so that both row-wise 16-byte reads
// (16 consecutive rows, one chunk) and transposing 8-byte reads (4 consecutive
// rows x 64 bytes) spread over all 64 banks.
template <int D>
__device__ __forceinline__ int swz(int row) {
  if constexpr (D == 128) {
    return ((row & 3) << 2) | ((row >> 2) & 3);
  } else {
    return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
  }
}

// Byte offset of element (row, col) in a swizzled [rows][D] bf16 tile; col is a
// multiple of 4 and the returned address is valid for an 8-byte access (or a
// 16-byte one when col is a multiple of 8).
template <int D>
__device__ __forceinline__ int tile_off(int row, int col) {
  const int chunk = (col >> 3) ^ swz<D>(row);
  return row * (D * 2) + chunk * 16 + (col & 7) * 2;
}

__device__ __forceinline__ bf16x8 lds_read_b128(const char* base, int off) {
  return *reinterpret_cast<const bf16x8*>(base + off);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes the
// addresses name a 4 x 16 block of 16-bit elements (lane i: row i/4, columns
// 4*(i%4)..+3); lane i receives column i of that block (4 elements, rows 0..3).
__device__ __forceinline__ s16x4 lds_read_tr(const char* base, int off) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(base + off));
}

// The same two reads at an LDS byte address held as an integer (base + immediate offset).
__device__ __forceinline__ bf16x8 lds_read_b128_at(uint32_t addr) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(addr);
}
__device__ __forceinline__ s16x4 lds_read_tr_at(uint32_t addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<__attribute__((address_space(3))) s16x4*>(addr));
}

__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// Value held by the lane 32 away (lane l <-> l^32).
__device__ __forceinline__ float other_half(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0] = {low half, low half}, r[1] = {high half, high half}
  const uint32_t lo = r[0], hi = r[1];
  const uint32_t o = (threadIdx.x & 32) ? lo : hi;
  return __builtin_bit_cast(float, o);
}

// max / sum over the lane pair (l, l^32); every lane gets the result.
__device__ __forceinline__ float pair_max(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t lo = r[0], hi = r[1];
  return fmaxf(__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi));
}
__device__ __forceinline__ float pair_sum(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t lo = r[0], hi = r[1];
  return __builtin_bit_cast(float, lo) + __builtin_bit_cast(float, hi);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 to_bf16x8(f32x8 v) { return __builtin_convertvector(v, bf16x8); }
__device__ __forceinline__ bf16x4 to_bf16x4(f32x4 v) { return __builtin_convertvector(v, bf16x4); }

// Stores a wavefront's 32 x D fp32 tile, held in the 32x32 MFMA accumulator layout (lane: row
// lane & 31; register q4*4 + e of block db: column db*32 + q4*8 + 4*(lane >> 5) + e), as bf16
// rows.  The tile is turned through 32*D*2 bytes of LDS that belong to the wavefront (16-byte
// chunk x of row r kept at chunk x ^ (r mod chunks-per-row)), so that every store instruction
// writes complete rows instead of 16 bytes of each of 32 rows.  mul scales this lane's row;
// dst points at row 0 of the tile (first column of the head); rows >= rows_valid are not
// written.  A wavefront's LDS accesses complete in program order, so only the compiler has
// to be kept from moving the reads over the writes.
template <int D>
__device__ __forceinline__ void store_tile_rows(char* turn, const f32x16 (&acc)[D / 32], float mul,
                                                __bf16* dst, size_t row_stride, int rows_valid) {
  constexpr int CPR = D / 8, RB = D * 2;
  const int lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      f32x4 a;
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] = acc[db][q4 * 4 + e] * mul;
      *reinterpret_cast<bf16x4*>(turn + c * RB + (((db * 4 + q4) ^ (c & (CPR - 1))) << 4) + 8 * g) = to_bf16x4(a);
    }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int rr = lane / CPR, cx = lane % CPR;
#pragma unroll
  for (int i = 0; i < 32 * CPR / 64; ++i) {
    const int r = i * (64 / CPR) + rr;
    const u32x4 w = *reinterpret_cast<const u32x4*>(turn + r * RB + ((cx ^ (r & (CPR - 1))) << 4));
    if (r < rows_valid) *reinterpret_cast<u32x4*>(dst + (size_t)r * row_stride + cx * 8) = w;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// ---- direct global -> LDS loads, issued as inline assembly ------------------
// The compiler orders every LDS read that follows a compiler-visible LDS-writing load
// behind a full vmcnt(0) wait, which would expose the whole global latency each tile.
// Issued as assembly the loads stay in flight across the tile's LDS reads; the kernels
// wait for them explicitly (wait_vmcnt) before the barrier that publishes the tile.
// Lane L's bytes land at lds_addr + L*size; lds_addr and base are wave-uniform, the
// global address is base + byte_off (32-bit unsigned, per lane).  Extra outstanding
// loads the compiler does not know of can only make its own vmcnt waits stricter.
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ __forceinline__ void lds_dma16(const void* base, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}
__device__ __forceinline__ void lds_dma4(const void* base, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :: "s"(lds_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}
// A pointer the compiler cannot prove wave-uniform (it depends on the wave index), moved
// to scalar registers.
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
  const uint64_t u = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
template <int V>
struct IntC { static constexpr int value = V; };
// Marks a loaded operand as used here, so that the compiler waits for its global load at
// this point (before the main loop) instead of keeping conservative vmcnt waits inside
// the loop, where they would also wait for the direct-to-LDS loads in flight.
__device__ __forceinline__ void settle(const bf16x8& x) { asm volatile("" :: "v"(x)); }

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ---- MFMAs issued as assembly, for kernels that need more than 256 registers -------------
// In such a kernel the compiler gives every MFMA it selects an AGPR destination and then
// copies each score to a VGPR (VALU cannot read AGPRs).  Score MFMAs are therefore written as
// assembly with a VGPR destination and the loop-invariant B operand in an AGPR tuple (which
// an MFMA may read directly).  The compiler does not know that the statement is an MFMA, so
// it inserts no wait states for readers of d: every reader must be at least two MFMAs
// downstream in program order (tests/test_isa_hazards.py checks the emitted assembly for it).
__device__ __forceinline__ void mfma32_v(f32x16& d, const bf16x8& a, const bf16x8& b, bool first) {
  if (first) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
// The same with three register tuples passed through unchanged.  Volatile statements keep
// their program order, so arithmetic that reads f0/f1/f2 after this call cannot be moved
// before the MFMA, and arithmetic that produced them cannot be moved after it: this is how
// the VALU work is spread evenly between the MFMAs.
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ void mfma32_v(f32x16& d, const bf16x8& a, const bf16x8& b, bool first,
                                         f32x16& f0, f32x16& f1, u32x8& f2) {
  if (first) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %4, %5, 0"
                          : "=&v"(d), "+v"(f0), "+v"(f1), "+v"(f2) : "v"(a), "a"(b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %4, %5, %0"
                    : "+v"(d), "+v"(f0), "+v"(f1), "+v"(f2) : "v"(a), "a"(b));
}

// Rebinds a loaded operand to an AGPR tuple (and, like settle(), makes the compiler wait
// for its global load here).
__device__ __forceinline__ void to_agpr(bf16x8& x) { asm volatile("" : "=a"(x) : "0"(x)); }

// Accumulation as assembly: accumulator in an AGPR tuple, both operands in VGPRs; the tuples
// are passed through unchanged (see mfma32_v).  Readers of acc other than the next
// accumulation into it must wait out the MFMA themselves.
__device__ __forceinline__ void mfma32_acc(f32x16& acc, const bf16x8& a, const bf16x8& b,
                                           f32x16& f0, f32x16& f1, u32x8& f2) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %4, %5, %0"
               : "+a"(acc), "+v"(f0), "+v"(f1), "+v"(f2) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma32_acc(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// Wait states after assembly MFMAs, before code the compiler generates reads their results (it
// does not know they were MFMA results).  The tuples are passed through, so that their readers
// cannot be scheduled above the wait.
__device__ __forceinline__ void wait_mfma_v(f32x16& a) {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(a));
}
__device__ __forceinline__ void wait_mfma_v(f32x16& a, f32x16& b) {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void wait_mfma_a(f32x16& a, f32x16& b, f32x16& c, f32x16& d) {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" : "+a"(a), "+a"(b), "+a"(c), "+a"(d));
}

// ---- kernel launch ----------------------------------------------------------
// Every kernel of the library is launched through hipLaunchKernel, whose return value is that
// launch's own status.  The thread's sticky "last error" is neither read nor cleared, so an
// error other code left pending in the runtime stays where it is and is never mistaken for
// the library's.
template <class... P, size_t... I>
inline hipError_t launch_impl(void (*kern)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                              std::tuple<P...>& vals, std::index_sequence<I...>) {
  void* ptrs[] = {static_cast<void*>(const_cast<std::remove_const_t<std::tuple_element_t<I, std::tuple<P...>>>*>(
      &std::get<I>(vals)))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kern), grid, block, ptrs, lds, stream);
}
template <class... P, class... A>
inline hipError_t launch(void (*kern)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                         const A&... args) {
  static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
  std::tuple<P...> vals{static_cast<P>(args)...};
  return launch_impl(kern, grid, block, lds, stream, vals, std::index_sequence_for<P...>{});
}

// ---- launchers (defined next to their kernels) -----------------------------
// The RoPE launchers work on the tokens [tab.cu[0], tab.cu[tab.n]) of the clips in tab.
hipError_t launch_rope3d(void* x, const RopeTable& tab, int n_heads, int head_dim,
                         int dim_t, int dim_h, int dim_w, float theta, int inverse,
                         hipStream_t stream);

hipError_t launch_qknorm_rope3d(const void* x, void* y, const float* gain, float eps,
                                const RopeTable& tab, int n_heads, int head_dim,
                                int dim_t, int dim_h, int dim_w, float theta, hipStream_t stream);

hipError_t launch_qknorm_rope3d_bwd(const void* x, const void* dy, void* dx, const float* gain,
                                    float eps, float* dgain, const RopeTable& tab,
                                    int n_heads, int head_dim, int dim_t, int dim_h, int dim_w,
                                    float theta, hipStream_t stream);   // accumulates into dgain
hipError_t launch_zero_f32(float* p, int n, hipStream_t stream);

hipError_t launch_tattn_fwd(const void* q, const void* k, const void* v, const TemporalTable& tab,
                            int n_heads, int head_dim, float scale, void* out, hipStream_t stream);

hipError_t launch_tattn_bwd(const void* q, const void* k, const void* v, const void* dout,
                            const TemporalTable& tab, int n_heads, int head_dim, float scale, void* dq,
                            void* dk, void* dv, hipStream_t stream);

// FP8 path.  scales: the q row exponents and the units' scale words (fp8_scales_bytes() bytes).
hipError_t launch_fp8_pack_q(const void* q, int total, int n_heads, int head_dim, float pre, void* q8,
                             void* scales, hipStream_t stream);
hipError_t launch_fp8_pack_kv(const void* k, const void* v, const Fp8ClipTable& clips, int n_units, int total,
                              int n_heads, int head_dim, void* k8, void* vT8, void* scales, hipStream_t stream);
hipError_t launch_attn_fwd_fp8(const void* q8, const void* k8, const void* vT8, const void* scales,
                               const Fp8SegTable& segs, int n_units, int total, int n_heads, int head_dim,
                               void* out, float* lse, hipStream_t stream);
size_t fp8_scales_bytes(int total, int n_heads, int n_units);

// Segs is SegTable (self-attention) or XSegTable (cross-attention); total_q is the number
// of query tokens (rows of lse, Delta).
template <class Segs>
hipError_t launch_attn_fwd(const void* q, const void* k, const void* v, const Segs& segs,
                           int total_q, int n_heads, int head_dim, float scale, void* out,
                           float* lse, hipStream_t stream);

// Once per call: the statistics of all total_q query tokens.
hipError_t launch_bwd_prepare(const void* out, const void* dout, const float* lse, float* delta, float* lse2,
                              float* sentinel, int total_q, int n_heads, int head_dim, hipStream_t stream);
// The sequences of segs (one run of a call's clips).  dkv32: optional fp32 dK, dV accumulators of
// total_kv rows each (query-split pass); [kv_lo, kv_hi) is the run's range of key rows.
template <class Segs>
hipError_t launch_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                           const float* lse, const void* dout, const Segs& segs, int total_q,
                           int n_heads, int head_dim, float scale, void* dq, void* dk, void* dv,
                           float* delta, float* lse2, float* sentinel, float* dkv32, int total_kv,
                           int kv_lo, int kv_hi, hipStream_t stream);

}  // namespace vfm
