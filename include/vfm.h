/*
 * vfm.h -- C ABI of libvfm: packed 3D-RoPE multi-head self-attention for video
 * diffusion transformers on AMD MI355X (gfx950), forward and backward.
 *
 * The operations are the hot path of the paper's video foundation model runs
 * (arxiv 2503.12964):
 *   - Section 3.1: clips of different shapes are concatenated along the
 *     sequence dimension with micro-batch 1 (sequence packing).  Every tensor
 *     here is therefore packed as [total_tokens, n_heads, head_dim] and the
 *     clip boundaries are the prefix sums cu_seqlens[0..n_seqs].
 *   - Sections 4.2 and 4.6: a clip's 3D latent grid (T, H, W) is flattened to
 *     one token sequence, t slowest and w fastest.
 *   - Sections 4.4 and 4.6: full attention -- every query token is computed
 *     against the keys and values of all tokens of its own clip, bidirectional,
 *     never across clips.
 *   - Section 5.2, Table 1: multi-head attention, head_dim 128.
 * The rotary embedding, the softmax scale and the log-sum-exp units are not
 * given by the paper; the definitions used are stated at each entry point.
 *
 * Conventions common to all entry points
 *   - Tensor arguments are DEVICE pointers to contiguous memory, 16-byte
 *     aligned, owned by the caller.  The library never allocates, frees or
 *     synchronises; it only enqueues kernels on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = the default stream).  Buffers must stay alive
 *     until that work has completed.
 *   - cu_seqlens and thw are HOST int32 arrays, read before the call returns
 *     (they fix the launch geometry and travel to the kernels by value).
 *   - Element type is bf16 (VFM_BF16).  Accumulation is fp32.
 *   - head_dim is 64 or 128.  Empty clips (cu_seqlens[s] == cu_seqlens[s+1]) are
 *     legal and do no work.  n_seqs is not limited (Section 3.1 packs images and
 *     videos together, and the spatial view of Section 4.6 makes every latent
 *     frame a sequence): the clip tables travel to the kernels by value and hold
 *     VFM_MAX_SEQS clips, so a call with more is cut, inside the library, into
 *     consecutive launches on hip_stream over runs of VFM_MAX_SEQS clips in
 *     packed order (VFM_MAX_XSEQS sequences for cross-attention).  Clips are
 *     independent, so the result does not depend on where the runs are cut.
 *   - Every function returns a vfm_status; 0 is success.  Argument errors are
 *     detected before anything is launched and leave all outputs untouched.
 *   - Re-entrant: no global mutable state (beyond the calling thread's last
 *     launch error, see vfm_last_hip_error).
 *   - The library uses the HIP runtime (libamdhip64) of the process it is
 *     loaded into, and that must be the runtime that owns the pointers and
 *     the stream handed over.  A process that holds two copies of the runtime
 *     (for example a framework that ships its own, loaded AFTER this library
 *     had already pulled in the system's) gets VFM_ERR_LAUNCH, "no ROCm-capable
 *     device is detected": load the framework first.
 */
#ifndef VFM_H
#define VFM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VFM_MAX_SEQS 256    /* clips per launch (run), self-attention, RoPE, temporal attention */
#define VFM_MAX_XSEQS 128   /* sequences per launch (run), cross-attention */
#define VFM_NOALLOC_MAX_ROWS (1 << 21) /* n_heads * total_tokens, vfm_attn_bwd_noalloc */

#define VFM_API __attribute__((visibility("default")))

typedef enum {
  VFM_OK = 0,
  VFM_ERR_NULL = 1,        /* a required pointer is NULL */
  VFM_ERR_SHAPE = 2,       /* total_tokens/n_heads/head_dim/n_seqs/scale/theta/eps out of range */
  VFM_ERR_CU_SEQLENS = 3,  /* not starting at 0, decreasing, or not ending at total_tokens */
  VFM_ERR_THW = 4,         /* T*H*W differs from the clip length, or a non-positive extent */
  VFM_ERR_SPLIT = 5,       /* dim_t+dim_h+dim_w != head_dim, or an odd/negative part */
  VFM_ERR_DTYPE = 6,       /* unsupported element type */
  VFM_ERR_WORKSPACE = 7,   /* workspace NULL, misaligned or too small */
  VFM_ERR_LAUNCH = 8,      /* the HIP runtime refused a launch */
  VFM_ERR_ALIGN = 9,       /* a tensor pointer is not 16-byte aligned */
  VFM_ERR_SCRATCH = 10     /* sizes beyond the built-in scratch of vfm_attn_bwd_noalloc */
} vfm_status;

typedef enum { VFM_BF16 = 0, VFM_F32 = 1 /* not implemented: VFM_ERR_DTYPE */ } vfm_dtype;

/*
 * 3D rotary position embedding, in place, on x[total_tokens, n_heads, head_dim]
 * (applied to q and to k before attention).
 *
 * Token n of clip s has local index r = n - cu_seqlens[s] and grid position
 * t = r / (H*W), h = (r / W) % H, w = r % W with (T,H,W) = thw[3s..3s+2]
 * (flatten order of Sections 4.2/4.6).  The head vector is cut into three
 * contiguous slices of widths dim_t, dim_h, dim_w.  In the slice of axis A
 * (width d_A, position p_A) the adjacent pair (x[2i], x[2i+1]), i < d_A/2, is
 * rotated by phi = p_A * theta^(-2i/d_A):
 *     x[2i]'   = x[2i] cos(phi) - x[2i+1] sin(phi)
 *     x[2i+1]' = x[2i] sin(phi) + x[2i+1] cos(phi)
 * inverse != 0 rotates by -phi (the transpose; carries gradients back).
 * The angle is formed and range-reduced in fp64, sin/cos and the products are
 * fp32, and the result is rounded to bf16 (nearest even).
 *
 * thw: host [n_seqs,3]; cu_seqlens: host [n_seqs+1].
 * Errors: NULL, SHAPE, CU_SEQLENS, THW, SPLIT, DTYPE, ALIGN, LAUNCH.
 */
VFM_API int vfm_rope3d(void* x, const int32_t* thw, const int32_t* cu_seqlens, int n_seqs,
               int total_tokens, int n_heads, int head_dim,
               int dim_t, int dim_h, int dim_w, float theta, int inverse,
               vfm_dtype dt, void* hip_stream);

/*
 * Per-head normalisation of q or k fused with the 3D rotary embedding above, in one
 * pass over memory.  Section 4.5.1 normalises Q and K per attention head right
 * before attention; it is taken here as root-mean-square normalisation with a
 * learned gain shared by all heads.  For every token and head:
 *     r   = 1 / sqrt(mean_d x[d]^2 + eps)
 *     z_d = x[d] * r * gain[d]
 *     y   = rotation of z exactly as in vfm_rope3d
 * x, y: bf16 [total_tokens, n_heads, head_dim], y may be the same buffer as x
 * (in place); gain: device fp32 [head_dim]; eps >= 0.  Sums, r and the rotation
 * are fp32, y is rounded once to bf16.
 * Errors: NULL, SHAPE, CU_SEQLENS, THW, SPLIT, DTYPE, ALIGN, LAUNCH.
 */
VFM_API int vfm_qknorm_rope3d(const void* x, const float* gain, float eps, void* y,
                      const int32_t* thw, const int32_t* cu_seqlens, int n_seqs,
                      int total_tokens, int n_heads, int head_dim,
                      int dim_t, int dim_h, int dim_w, float theta,
                      vfm_dtype dt, void* hip_stream);

/*
 * Gradients of vfm_qknorm_rope3d.  With n = x r, given dy:
 *     dz      = transpose rotation of dy
 *     dgain_d = sum over tokens and heads of dz_d n_d
 *     dn      = dz * gain
 *     dx      = r * (dn - n * mean_d(dn_d n_d))
 * x is the forward's input (r is recomputed from it, nothing is saved by the
 * forward).  dx: bf16, fully overwritten; it may be the same buffer as dy, never
 * the same as x (SHAPE).  dgain: device fp32 [head_dim], overwritten (zeroed by
 * this call, then accumulated with fp32 atomics, so its last bits may differ
 * from run to run; dx is bitwise reproducible).
 * Errors: NULL, SHAPE, CU_SEQLENS, THW, SPLIT, DTYPE, ALIGN, LAUNCH.
 */
VFM_API int vfm_qknorm_rope3d_bwd(const void* x, const float* gain, float eps, const void* dy,
                          void* dx, float* dgain,
                          const int32_t* thw, const int32_t* cu_seqlens, int n_seqs,
                          int total_tokens, int n_heads, int head_dim,
                          int dim_t, int dim_h, int dim_w, float theta,
                          vfm_dtype dt, void* hip_stream);

/*
 * Attention forward.  For every clip [a,b) and head h:
 *     S_ij  = scale * sum_d q[i,h,d] k[j,h,d]          i, j in [a,b)
 *     out_i = sum_j softmax_j(S_ij) v[j,h,:]
 *     lse_i = ln sum_j exp(S_ij)                        (natural log)
 * q, k, v, out: bf16 [total_tokens, n_heads, head_dim]; lse: fp32
 * [n_heads, total_tokens].  out and lse are fully overwritten for every token
 * of a non-empty clip.  The result is bitwise reproducible from run to run.
 * Errors: NULL, SHAPE, CU_SEQLENS, DTYPE, ALIGN, LAUNCH.
 */
VFM_API int vfm_attn_fwd(const void* q, const void* k, const void* v,
                 const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                 int n_heads, int head_dim, float scale,
                 void* out, float* lse, vfm_dtype dt, void* hip_stream);

/*
 * Bytes of device workspace vfm_attn_bwd needs for these sizes (0 if the sizes
 * are invalid).  The workspace holds Delta_i = sum_d dout[i,h,d] out[i,h,d] and
 * lse * log2(e) (two fp32 [n_heads, total_tokens] arrays, each padded to 256
 * bytes) followed by 256 bytes of constants the kernels read for rows past a
 * clip's end; its contents need not be initialised and are garbage afterwards.
 */
VFM_API size_t vfm_attn_bwd_workspace_size(int total_tokens, int n_heads, int head_dim);

/*
 * Attention backward: gradients of sum(out * dout) with respect to q, k, v,
 * given the forward's out and lse (no gradient flows into lse):
 *     P_ij   = exp(S_ij - lse_i)
 *     dv_j   = sum_i P_ij dout_i
 *     dS_ij  = P_ij (sum_d dout[i,d] v[j,d] - Delta_i)
 *     dq_i   = scale * sum_j dS_ij k_j
 *     dk_j   = scale * sum_i dS_ij q_i
 * dq, dk, dv: bf16 [total_tokens, n_heads, head_dim], fully overwritten (not
 * accumulated into).  workspace: device, 256-byte aligned, at least
 * vfm_attn_bwd_workspace_size() bytes.  No atomics are used: dq, dk and dv are
 * bitwise reproducible from run to run.
 * Accuracy: Delta_i = sum_d dout[i,d] out[i,d] is formed from the bf16 `out`
 * handed in, whose rounding (2^-9 relative) is harmless once a clip has a few
 * dozen keys (|out| shrinks like 1/sqrt(keys)) but would reach several percent
 * of dq, dk in clips of two to eight tokens, where dS cancels almost completely.
 * For clips of at most 32 keys the library therefore recomputes Delta_i as
 * sum_j P_ij (dout_i . v_j), the same quantity without the rounded `out`; with
 * it dq, dk, dv stay within 1.5e-2 relative RMS of the exact gradients for every
 * clip length.
 * Errors: NULL, SHAPE, CU_SEQLENS, DTYPE, ALIGN, WORKSPACE, LAUNCH.
 */
VFM_API int vfm_attn_bwd(const void* q, const void* k, const void* v, const void* out,
                 const float* lse, const void* dout, const int32_t* cu_seqlens,
                 int n_seqs, int total_tokens, int n_heads, int head_dim, float scale,
                 void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                 vfm_dtype dt, void* hip_stream);

/*
 * vfm_attn_bwd for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments (minus the workspace), same kernels and
 * bitwise the same dq, dk, dv as vfm_attn_bwd.  The statistics vfm_attn_bwd keeps
 * in its workspace live in an array built into the library's device code instead:
 * 2 * VFM_NOALLOC_MAX_ROWS * 4 + 256 bytes (16 MiB) that every GPU the library runs
 * on holds from the first use until the process ends.  Limit:
 * n_heads * total_tokens <= VFM_NOALLOC_MAX_ROWS (the 56,320-token, 32-head
 * latent fits); larger calls return VFM_ERR_SCRATCH and launch nothing.
 * The call allocates and frees nothing, on the device or through any library; it
 * looks up the array's device address once per device (the device that is
 * current at the call must be the one that owns the stream and the tensors) and
 * enqueues the kernels on hip_stream.  All calls on one GPU share that GPU's
 * array: calls that may overlap in time on one GPU (different streams, or
 * different threads) race on it and must be serialised by the caller; calls on
 * one stream are safe.  Nothing in the array has to be cleared between calls
 * (every call first rewrites what it later reads).
 * Errors: NULL, SHAPE, CU_SEQLENS, DTYPE, ALIGN, SCRATCH, LAUNCH.
 */
VFM_API int vfm_attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* out,
                         const float* lse, const void* dout, const int32_t* cu_seqlens,
                         int n_seqs, int total_tokens, int n_heads, int head_dim, float scale,
                         void* dq, void* dk, void* dv, vfm_dtype dt, void* hip_stream);

/*
 * Cross-attention forward (Section 4.2: in every transformer block the video
 * query tensor attends to the text embedding's keys and values).  Sequence s
 * owns queries [cu_seqlens_q[s], cu_seqlens_q[s+1]) of q[total_q, n_heads,
 * head_dim] and keys/values [cu_seqlens_kv[s], cu_seqlens_kv[s+1]) of
 * k, v[total_kv, n_heads, head_dim]:
 *     S_ij  = scale * sum_d q[i,h,d] k[j,h,d]
 *     out_i = sum_j softmax_j(S_ij) v[j,h,:],   lse_i = ln sum_j exp(S_ij)
 * out: bf16 [total_q, n_heads, head_dim]; lse: fp32 [n_heads, total_q].  Both
 * cu arrays are host int32 [n_seqs+1].  A sequence
 * with queries must have at least one key (CU_SEQLENS); one with keys and no
 * queries is legal.  Same kernels, arithmetic and reproducibility as
 * vfm_attn_fwd, which is the case of equal ranges.
 * Errors: NULL, SHAPE, CU_SEQLENS, DTYPE, ALIGN, LAUNCH.
 */
VFM_API int vfm_xattn_fwd(const void* q, const void* k, const void* v,
                  const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_kv, int n_seqs,
                  int total_q, int total_kv, int n_heads, int head_dim, float scale,
                  void* out, float* lse, vfm_dtype dt, void* hip_stream);

/*
 * Cross-attention backward: dq [total_q, ...], dk, dv [total_kv, ...] from dout,
 * with the formulas of vfm_attn_bwd, i over a sequence's queries and j over its
 * keys.  Keys of a sequence without queries get zero gradients.  workspace:
 * device, 256-byte aligned, at least vfm_xattn_bwd_workspace_size() bytes (the
 * statistics of vfm_attn_bwd plus fp32 dK, dV accumulators).  dq is written
 * once and is reproducible.  When the key ranges are short (few key tiles for
 * many queries) the query range is split over workgroups and dK, dV are summed
 * with fp32 atomics, so their last bits may differ from run to run; otherwise
 * they are written once as in vfm_attn_bwd.
 * Errors: NULL, SHAPE, CU_SEQLENS, DTYPE, ALIGN, WORKSPACE, LAUNCH.
 */
VFM_API size_t vfm_xattn_bwd_workspace_size(int total_q, int total_kv, int n_heads, int head_dim);
VFM_API int vfm_xattn_bwd(const void* q, const void* k, const void* v, const void* out,
                  const float* lse, const void* dout,
                  const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_kv, int n_seqs,
                  int total_q, int total_kv, int n_heads, int head_dim, float scale,
                  void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                  vfm_dtype dt, void* hip_stream);

/*
 * Temporal attention of the spatial-temporal transformer (Section 4.6): attention
 * among the inter-frame tokens of one pixel, i.e. the packed buffer [b, h*w*t, d]
 * read as [(b*h*w), t, d].  For clip s with grid (T,H,W) = thw[3s..3s+2] and
 * pixel p < H*W the sequence is the T rows cu_seqlens[s] + t*H*W + p; per head
 *     out_i = sum_j softmax_j(scale * q_i . k_j) v_j       i, j over the T frames.
 * Any T >= 1 (the section speaks of hundreds of frames): up to 32 frames a
 * sequence is one register tile and the call is bound by HBM; a call (run of
 * clips) in which some clip has more is walked in 32-frame blocks with an
 * online softmax.  q, k, v, out: bf16 [total_tokens, n_heads, head_dim]; thw,
 * cu_seqlens: host.  No statistics are saved.
 * Errors: NULL, SHAPE, CU_SEQLENS, THW, DTYPE, ALIGN, LAUNCH.
 */
VFM_API int vfm_tattn_fwd(const void* q, const void* k, const void* v,
                  const int32_t* thw, const int32_t* cu_seqlens, int n_seqs,
                  int total_tokens, int n_heads, int head_dim, float scale,
                  void* out, vfm_dtype dt, void* hip_stream);

/*
 * Temporal attention backward: dq, dk, dv (bf16, fully overwritten) from dout.
 * The softmax is recomputed from q and k; Delta_i = sum_j P_ij (dout_i . v_j).
 * No atomics, no workspace; every output is written once, except that with clips
 * of more than 32 frames the first 8 bytes of every dq row hold that query's
 * softmax statistics while the call runs, before dq is written over them.
 * Errors: NULL, SHAPE, CU_SEQLENS, THW, DTYPE, ALIGN, LAUNCH.
 */
VFM_API int vfm_tattn_bwd(const void* q, const void* k, const void* v, const void* dout,
                  const int32_t* thw, const int32_t* cu_seqlens, int n_seqs,
                  int total_tokens, int n_heads, int head_dim, float scale,
                  void* dq, void* dk, void* dv, vfm_dtype dt, void* hip_stream);

/*
 * FP8 attention forward (Section 5.2 reports FP8 multi-head attention for
 * inference).  Operands are 8-bit floats in the E4M3 format of the OCP 8-bit
 * floating point specification, with one power-of-two scale per tile, chosen by
 * vfm_fp8_pack, which prepares the operands once per (q, k, v):
 *   tile          = a (token, head) row of q  |  a (head, unit) of k  |  a (head, unit) of v
 *                   (a "unit" is 64 consecutive keys of one clip, zero padded at
 *                   the clip's end; units are numbered clip by clip in packed
 *                   order, clip s owning ceil(len_s / 64))
 *   e             = the largest integer with  max|x| * 2^e <= 448  over the tile,
 *                   limited to [-120, 120], 0 for an all-zero tile
 *   x8            = round_to_nearest_even(x * 2^e)          (x is read back as x8 * 2^-e)
 * For q, x is q * scale * log2(e) rounded to fp32 (scale = the softmax scale):
 * the product q8 . k8, descaled, is then the softmax exponent in log2 units.
 * The kernel hands 2^-e of both tiles to the matrix instruction as its
 * block-scale inputs, which applies them exactly and at no cost.  The fourth
 * tensor of the row, P, is scaled per query row by the softmax reference point
 * (every probability is stored relative to it) times a fixed 2^6.
 * Packed buffers, per head h:
 *   q8  [n_heads][total_tokens][head_dim]
 *   k8  [n_heads][units][64][head_dim]: key row r of a unit holds its 16-byte
 *       chunk c at chunk position c ^ ((r >> 1) & 7) (head_dim 128) or
 *       c ^ ((r >> 2) & 3) (head_dim 64)
 *   vT8 [n_heads][units][head_dim][64]: row d holds, at 16-byte chunk position
 *       c ^ ((d >> 2) & 3), the logical chunk c of a 64-byte row whose byte
 *       32 g + j (g < 2, j < 32) is key  32 (j / 16) + 8 ((j % 16) / 4) + 4 g + j % 4
 *       of the unit.
 *   scales: [n_heads][total_tokens] bytes 127 - e of the q rows, padded to a
 *       multiple of 256 bytes, then [n_heads][units] 32-bit words whose byte 0
 *       is 127 - e of the k unit and byte 1 is 127 - e of the v unit (bytes 2
 *       and 3 are 127).
 * (The chunk permutations are the kernels' LDS bank swizzle, the byte order is
 * the order the matrix instruction consumes keys in; callers treat the buffers
 * as opaque.)  vfm_fp8_pack_sizes returns the four sizes in bytes.
 * Errors: NULL, SHAPE (incl. a packed buffer beyond 4 GiB), CU_SEQLENS, DTYPE,
 * ALIGN, LAUNCH.
 */
VFM_API int vfm_fp8_pack_sizes(const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                       int n_heads, int head_dim,
                       size_t* q8_bytes, size_t* k8_bytes, size_t* vT8_bytes, size_t* scales_bytes);
VFM_API int vfm_fp8_pack(const void* q, const void* k, const void* v,
                 const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                 int n_heads, int head_dim, float scale,
                 void* q8, void* k8, void* vT8, void* scales, vfm_dtype dt, void* hip_stream);

/*
 * out, lse as vfm_attn_fwd, computed from the packed E4M3 operands with FP8
 * matrix instructions and fp32 accumulation (q', k', v' = the values the tiles
 * read back as):
 *     S_ij  = ln(2) * sum_d q'[i,d] k'[j,d]        (= scale q_i . k_j up to rounding)
 *     out_i = sum_j softmax_j(S_ij) v'[j,:]
 * The probabilities are rounded to E4M3 (3 mantissa bits) before the second
 * product, so out carries a relative error of a few percent against the exact
 * result on the same quantised operands; lse is accumulated in fp32.  out: bf16
 * [total_tokens, n_heads, head_dim]; lse: fp32 [n_heads, total_tokens].
 * Errors: NULL, SHAPE, CU_SEQLENS, ALIGN, LAUNCH.
 */
VFM_API int vfm_attn_fwd_fp8(const void* q8, const void* k8, const void* vT8, const void* scales,
                     const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                     int n_heads, int head_dim,
                     void* out, float* lse, void* hip_stream);

/*
 * The tile scheduler, on the host (nothing is launched): which rows each
 * workgroup of a launch takes.  Section 3.1's packed clips are cut into tiles of
 * rows_per_tile rows that never straddle a clip (so blocks between different
 * clips are never enumerated), clips longest first, and the (head, tile) units
 * are dealt to the grid so that the workgroups of one XCD (workgroup index mod
 * 8) take consecutive tiles of the same head.  The attention kernels use this
 * very mapping over query rows with rows_per_tile = 256 in the dQ kernel and
 * vfm_attn_fwd_tile_rows() in the forward, and over key rows with 128 (dK/dV).
 * (A backward launch at head_dim 128 whose sequences all have at most 1,024
 * rows deals both kinds of tile from one grid, per (head, sequence) the key
 * tiles and then the query tiles, with the same tile heights and XCD rule.)
 * For workgroup b < *n_blocks: units[3b] = head (-1: the workgroup is grid
 * padding and exits), units[3b+1] = first packed row, units[3b+2] = rows
 * (1..rows_per_tile).  With more than VFM_MAX_SEQS clips the call is one launch
 * per run of VFM_MAX_SEQS clips; the grids of the launches follow one another in
 * units (each a multiple of 8 workgroups).  units is a HOST int32 [capacity][3]
 * array; *n_blocks is always set; SHAPE if capacity < *n_blocks.
 */
VFM_API int vfm_schedule_units(const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                       int n_heads, int rows_per_tile, int32_t* units, int capacity,
                       int* n_blocks);

/*
 * Query rows per workgroup that vfm_attn_fwd uses for run `run` (0-based; a call
 * with at most VFM_MAX_SEQS clips has the single run 0) of these clips, on the
 * host: 256 at head_dim 128 when the run's longest clip has more than 1,024
 * tokens, otherwise 128 (two workgroups per compute unit, whose prologues and
 * epilogues overlap each other's loops); always 128 at head_dim 64.
 * Errors: NULL, SHAPE (also: no such run), CU_SEQLENS.
 */
VFM_API int vfm_attn_fwd_tile_rows(const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                           int head_dim, int run, int* rows_per_tile);

/* Static, human-readable text for a vfm_status. */
VFM_API const char* vfm_strerror(int status);

/* The HIP runtime's text for the error behind the calling thread's most recent
 * VFM_ERR_LAUNCH ("no error" if there was none).  Errors that other code left
 * pending in the runtime before a call into this library are discarded by the
 * library and never reported as its own. */
VFM_API const char* vfm_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* VFM_H */
