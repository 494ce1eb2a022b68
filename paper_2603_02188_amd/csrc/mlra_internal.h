// Internal helpers shared by the HIP sources of libmlra (not part of the public ABI).
#pragma once

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "mlra.h"

namespace mlra {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

// ---- element conversion ---------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round-to-nearest-even; NaN stays NaN (quiet).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float load_f32(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_f32(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void store_f32(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_f32(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// ---- context split plan -------------------------------------------------------------------------
// Context is cut into n_splits chunks of chunk_tokens (a multiple of 64) per (sequence, block).
struct SplitPlan {
  int n_splits;       // partial slots per (sequence, block) = grid extent over chunks
  int chunk_tokens;   // uniform chunk length
  int target_chunks;  // > 0: chunk lengths may follow the sequence lengths so that about this many chunks
                      // per block are active in total (see launch_plan_chunks); 0: uniform chunks only
  bool single_if_uniform = false;   // with target_chunks: a batch of nearly equal lengths is not cut at all
};

int device_cu_count();

// Kernel attributes (the dynamic LDS limit) belong to a device: a launcher sets them the first time it
// runs on each device.  needed() says whether the current device still lacks them, done() records that
// they are set.  Two threads racing through a first call both set the attributes, which is harmless.
class PerDeviceSetup {
 public:
  bool needed(int* dev) const {
    if (hipGetDevice(dev) != hipSuccess || *dev < 0 || *dev >= 64) { *dev = -1; return true; }
    return ((seen_.load(std::memory_order_acquire) >> *dev) & 1ull) == 0;
  }
  void done(int dev) {
    if (dev >= 0) seen_.fetch_or(1ull << dev, std::memory_order_release);
  }
 private:
  std::atomic<unsigned long long> seen_{0};
};
SplitPlan plan_splits(int batch, int n_blocks, int max_seq_len);

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- launchers implemented in the kernel sources -----------------------------------------------
// Optional timing of one kernel.  With both events set, a launch through MLRA_LAUNCH_TIMED records the
// kernel's own start and end into them (the interval a kernel trace reports as its duration), not stream
// markers around it, which would add the marker packets' own latency to short kernels.
struct KernelTimer {
  hipEvent_t start = nullptr, stop = nullptr;
  bool on() const { return start && stop; }
};
#define MLRA_LAUNCH_TIMED(timer, kernel, grid, block, lds, stream, ...)                                       \
  do {                                                                                                        \
    if ((timer).on())                                                                                         \
      hipExtLaunchKernelGGL(HIP_KERNEL_NAME(kernel), grid, block, lds, stream, (timer).start, (timer).stop, 0, \
                            __VA_ARGS__);                                                                     \
    else                                                                                                      \
      hipLaunchKernelGGL(HIP_KERNEL_NAME(kernel), grid, block, lds, stream, __VA_ARGS__);                     \
  } while (0)

struct DecodeArgs {
  const void* latent;
  const void* rope;
  const int32_t* page_table;
  const int32_t* seq_lens;
  int page_size, max_pages, n_blocks, d_cb, d_r;
  int batch, h, d_h;   // h: heads served by one block (all heads, or the heads of one group)
  int groups;          // 1: every block serves every head (Eq. (5)); 2: block b serves the heads of group
                       //    b / (n_blocks / 2) only (Eq. (6)); q_rope and out then hold groups * h heads
  const void* q_abs;
  const void* q_rope;
  const void* w_uv;
  float softmax_scale, out_scale;
  void* out;
  int out_dtype;
  float* lse;
  const void* gate;    // optional [batch][groups * h][d_h] of the cache dtype: out is multiplied by it elementwise
  float* part_z;   // [batch][n_blocks][n_splits][h][d_cb]
  float* part_ml;  // [batch][n_blocks][n_splits][h][2]  (running max, running sum)
  int q_group;         // > 1: entries [i q_group, (i + 1) q_group) of the batch are the query tokens of one sequence
  int32_t* seq_order;  // [batch] sequence ids, longest first (workspace); filled by the MFMA launcher when used
  int32_t* chunk_tab;  // [batch] per-sequence chunk length (workspace); filled by launch_plan_chunks when used
  int32_t* unit_tab;   // [batch * n_splits] active (sequence, chunk) pairs, then -1 (workspace); same
  bool balanced;       // chunk lengths follow the sequence lengths (chunk_tab) instead of plan.chunk_tokens
  bool rows_bf16;      // the decode kernel writes each chunk's partial as a normalised bf16 row z / l (the MLRA
                       // MFMA kernels); otherwise fp32 partials Z (the MLA and the generic kernels)
  SplitPlan plan;
  int dtype;
  hipStream_t stream;
  KernelTimer t_main, t_epi;   // set by mlra_kernel_timing_begin: the decode kernel and the merge / up-projection
};

// Factor that takes the raw score to the log2 domain: tau log2(e), or 1 when the caller's queries already
// carry it (softmax_scale == MLRA_SCALE_FOLDED, see mlra_absorb_q_folded).
inline float softmax_scale_log2(float softmax_scale) {
  return softmax_scale == MLRA_SCALE_FOLDED ? 1.0f : softmax_scale * 1.4426950408889634f;
}

int launch_append_kv(const mlra_cache* c, int batch, const void* c_kv_new, const void* k_rope_new, int src_dtype,
                     const int32_t* positions, hipStream_t stream);
// (h: heads per block; q_nope holds groups * h heads, block b reads those of group b / (n_blocks / groups))
// fold: factor on the absorbed queries before rounding; q_rope_out non-null: also q_rope_out = fold * q_rope
// ([batch][groups * h][d_r]), in the same launch
int launch_absorb_q_generic(int batch, int h, int d_h, int n_blocks, int groups, int d_cb, const void* q_nope,
                            const void* w_uk, void* q_abs, int dtype, hipStream_t stream, float fold = 1.f,
                            const void* q_rope = nullptr, void* q_rope_out = nullptr, int d_r = 0);
int launch_decode_generic(const DecodeArgs& a);
// seq_lens_out[s * q_len + j] = max(0, seq_lens[s] - (q_len - 1 - j)); page_table_out row s * q_len + j = row s
int launch_expand_queries(const int32_t* seq_lens, const int32_t* page_table, int batch, int q_len, int max_pages,
                          int32_t* seq_lens_out, int32_t* page_table_out, hipStream_t stream);
int launch_merge_upproj_generic(const DecodeArgs& a);

// Fast paths (bf16, MFMA); the *_supported predicates are false outside the shapes they were written for.
int launch_seq_order(const DecodeArgs& a);
int launch_plan_chunks(const DecodeArgs& a);
bool mla_mfma_supported(const DecodeArgs& a);
int launch_mla_mfma(const DecodeArgs& a);
bool decode_mfma_supported(const DecodeArgs& a);
bool decode_mfma_paired(int h, int n_blocks);
bool decode_gla_supported(const DecodeArgs& a);   // 256-channel latent heads (GLA-2)
int launch_decode_gla(const DecodeArgs& a);   // two blocks x 64 heads per workgroup instead of one x 128
int launch_decode_mfma(const DecodeArgs& a);
bool absorb_q_mfma_supported(int d_h, int d_cb, int dtype);
int launch_absorb_q_mfma(int batch, int h, int d_h, int n_blocks, int groups, int d_cb, const void* q_nope,
                         const void* w_uk, void* q_abs, hipStream_t stream, float fold = 1.f,
                         const void* q_rope = nullptr, void* q_rope_out = nullptr, int d_r = 0);   // d_r % 8 == 0
bool merge_upproj_mfma_supported(const DecodeArgs& a);
int launch_merge_upproj_mfma(const DecodeArgs& a);

struct GqaArgs {
  const void* k_pool;
  const void* v_pool;
  const int32_t* page_table;
  const int32_t* seq_lens;
  int page_size, max_pages, batch, h, g, d_h, dtype;
  const void* q;
  float softmax_scale;
  void* out;
  int out_dtype;
  float* part_o;   // [batch][n_splits][h][d_h]
  float* part_ml;  // [batch][n_splits][h][2]
  SplitPlan plan;
  hipStream_t stream;
};
int launch_gqa_generic(const GqaArgs& a);
bool gqa_mfma_supported(const GqaArgs& a);
int launch_gqa_mfma(const GqaArgs& a);
int launch_gqa_merge(const GqaArgs& a);

// ---- pre-attention of the new token (pre_attn.hip) ----------------------------------------------
// Weight matrices that share their rows (the K dimension) and sit side by side in the output.
struct GemmSegments {
  const void* w[3];
  int cols[3];      // columns of each matrix (= its leading dimension)
  int out_col[3];   // first output column of each matrix
  int count;
};
struct PrePlan {
  int n1, n2;                 // output columns of the down- and of the up-projection
  bool mfma1, mfma2;
  int slices1, rows1;         // K slices of the down-projection and rows per slice
  int slices2, rows2;
  size_t off_part1, off_cq, off_cs, off_part2, bytes;   // workspace layout
};
PrePlan pre_plan(int dtype, int batch, int d, int d_cq, int d_c, int d_r, int h, int d_h);
int launch_pre_attention(const mlra_cache* c, const mlra_pre_weights* w, int batch, const void* hidden,
                         const int32_t* positions, void* q_nope, void* q_rope, void* workspace,
                         hipStream_t stream);

static inline int check_launch() { return hipGetLastError() == hipSuccess ? MLRA_OK : MLRA_ERR_LAUNCH; }

}  // namespace mlra
