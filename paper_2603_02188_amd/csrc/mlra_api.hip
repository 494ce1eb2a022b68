// C ABI of libmlra: argument validation, context-split planning, workspace carving and dispatch.
#include <stdlib.h>

#include <vector>

#include "mlra_internal.h"

#include <algorithm>

namespace mlra {

// Optional per-kernel timing of the decode entry points (see mlra_kernel_timing_begin).
static std::vector<hipEvent_t> g_events;
static int g_timing_cap = 0, g_timing_calls = 0;

// four events per timed call: start / stop of the decode kernel, start / stop of the merge + up-projection
static bool timing_on() { return g_timing_calls < g_timing_cap; }
static KernelTimer timing_pair(int which) {
  KernelTimer t;
  if (timing_on()) {
    t.start = g_events[4 * g_timing_calls + 2 * which];
    t.stop = g_events[4 * g_timing_calls + 2 * which + 1];
  }
  return t;
}

int device_cu_count() {
  static std::atomic<int> cached[64];   // per device, 0 = not asked yet
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64) {
    const int have = cached[dev].load(std::memory_order_relaxed);
    if (have > 0) return have;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) {
      cached[dev].store(cus, std::memory_order_relaxed);
      return cus;
    }
  }
  (void)hipGetLastError();
  return 256;  // MI355X; used only when no device can be queried (e.g. sizing on a CPU-only host)
}

// Enough workgroups to cover every CU once when the batch alone cannot (the decode kernel runs one
// workgroup per CU, and each workgroup pays a fixed start-up and write-out cost), never chunks shorter
// than 128 tokens (a partial costs as much traffic as ~170 cached tokens of one block).
SplitPlan plan_splits(int batch, int n_blocks, int max_seq_len);

// Workgroups per (sequence, chunk): the MLRA kernels run one per latent block, the MLA kernel (one
// 512-dim latent) one per 64 heads.
static SplitPlan plan_decode(int batch, int h, int n_blocks, int d_cb, int max_seq_len) {
  int groups = (n_blocks == 1 && d_cb == 512) ? (h + 63) / 64 : n_blocks;
  if (d_cb == 128 && decode_mfma_paired(h, n_blocks)) groups = n_blocks / 2;   // two blocks per workgroup
  SplitPlan p = plan_splits(batch, groups, max_seq_len);
  // Split mode on the MFMA MLRA shape with long chunks: twice the chunk slots, so that long sequences of
  // a ragged batch can take more chunks than short ones (the decode entry decides per call whether it
  // uses them).  The planning kernel and the round of idle slots cost 6-9 us whatever the batch looks
  // like, and what they save depends on how ragged it is (about a tenth of the kernel for lengths spread
  // over a factor of two): chunks of 96 tiles or more (about 110 us of work) are where a ragged batch
  // gains more than a uniform one loses.
  if (d_cb == 128 && p.n_splits > 1 && p.chunk_tokens >= 6144 && 2 * p.n_splits * n_blocks <= 128) {
    p.target_chunks = p.n_splits * batch;
    p.n_splits *= 2;
  }
  // The forms that run one workgroup per two blocks or per 64 heads (MLRA-2 / GLA-2 at 128 heads, the MLA
  // baseline): when the batch alone gives about one round of workgroups, a ragged batch would leave the
  // CUs of its short sequences idle while the longest finishes.  Four chunk slots per sequence and a
  // target of two rounds let the planning kernel cut the long sequences and hand the chunks out longest
  // first; a batch of nearly equal lengths is left uncut.
  const bool mla = n_blocks == 1 && d_cb == 512;
  const bool two_per_wg = (d_cb == 128 && decode_mfma_paired(h, n_blocks)) || d_cb == 256;
  const long wgs = (long)batch * groups;
  if ((mla || two_per_wg) && p.n_splits == 1 && p.target_chunks == 0 && 2 * wgs > device_cu_count() &&
      wgs < 2 * device_cu_count() && max_seq_len >= 2048 && batch <= 512) {
    p.target_chunks = (int)std::max<long>(batch, 2L * device_cu_count() / groups);
    p.n_splits = 4;
    p.single_if_uniform = true;
  }
  return p;
}

SplitPlan plan_splits(int batch, int n_blocks, int max_seq_len) {
  const int kMinChunk = 128, kTile = 64;
  const long units = (long)batch * n_blocks;
  const long target = 1L * device_cu_count();
  long want = (target + units - 1) / units;
  const long max_splits = (max_seq_len + kMinChunk - 1) / kMinChunk;
  if (want > max_splits) want = max_splits;
  if (want < 1) want = 1;
  long chunk = (max_seq_len + want - 1) / want;
  chunk = (chunk + kTile - 1) / kTile * kTile;
  if (chunk < kMinChunk) chunk = kMinChunk;
  SplitPlan p;
  p.chunk_tokens = (int)chunk;
  p.n_splits = (int)((max_seq_len + chunk - 1) / chunk);
  if (p.n_splits < 1) p.n_splits = 1;
  p.target_chunks = 0;
  return p;
}

static bool valid_dtype(int d) { return d == MLRA_BF16 || d == MLRA_F32; }

// Scratch memory of mlra_decode_attn_static: one copy per GPU the library runs on, held until the process
// ends.  In host code the array's name is only a handle for the runtime; its device address on the
// current GPU comes from hipGetSymbolAddress, once per device, and that pointer is what the kernels get.
constexpr size_t kStaticScratchBytes = (size_t)MLRA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::atomic<void*> g_scratch_ptr[64];   // per device, null = not asked yet

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    (void)hipGetLastError();
    return MLRA_ERR_LAUNCH;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return MLRA_ERR_LAUNCH;
    }
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return MLRA_OK;
}

static size_t decode_ws_bytes(int batch, int h, int n_blocks, int d_cb, const SplitPlan& p) {
  const size_t units = (size_t)batch * n_blocks * p.n_splits;
  return align_up(units * h * d_cb * sizeof(float), 256) + align_up(units * h * 2 * sizeof(float), 256) +
         2 * align_up((size_t)batch * sizeof(int32_t), 256) +
         align_up((size_t)batch * p.n_splits * sizeof(int32_t), 256);
}

// h: heads served by one block (all heads when groups == 1, the heads of one group otherwise)
static int decode_common(const mlra_cache* c, int batch, int h, int groups, int d_h, const void* q_abs,
                         const void* q_rope, const void* w_uv, float softmax_scale, float out_scale, void* out,
                         int out_dtype, float* lse, void* workspace, size_t workspace_bytes, void* stream,
                         const void* gate = nullptr, int q_group = 1) {
  if (!c || !q_abs || !q_rope || !w_uv || !out) return MLRA_ERR_NULL;
  if (!c->latent || !c->rope || !c->page_table || !c->seq_lens) return MLRA_ERR_NULL;
  if (!valid_dtype(c->dtype) || !valid_dtype(out_dtype)) return MLRA_ERR_DTYPE;
  if (batch <= 0 || h <= 0 || d_h <= 0 || c->n_blocks <= 0 || c->d_cb <= 0 || c->d_r <= 0 || c->page_size <= 0 ||
      c->max_pages_per_seq <= 0 || c->num_pages <= 0)
    return MLRA_ERR_SHAPE;
  if ((long)c->max_pages_per_seq * c->page_size > 0x7fffffffL) return MLRA_ERR_SHAPE;
  if ((long)c->n_blocks * c->d_cb > 8192 || h * groups > 65535 || batch > 65535) return MLRA_ERR_SHAPE;
  if (c->n_blocks % groups != 0) return MLRA_ERR_SHAPE;
  const int max_seq_len = c->max_pages_per_seq * c->page_size;
  DecodeArgs a;
  a.plan = plan_decode(batch, h, c->n_blocks, c->d_cb, max_seq_len);
  const size_t need = decode_ws_bytes(batch, h, c->n_blocks, c->d_cb, a.plan);
  if (!workspace || workspace_bytes < need) return MLRA_ERR_WORKSPACE;
  if (((uintptr_t)workspace) % 256 != 0) return MLRA_ERR_WORKSPACE;
  const size_t units = (size_t)batch * c->n_blocks * a.plan.n_splits;
  a.part_z = (float*)workspace;
  a.part_ml = (float*)((char*)workspace + align_up(units * h * c->d_cb * sizeof(float), 256));
  a.seq_order = (int32_t*)((char*)a.part_ml + align_up(units * h * 2 * sizeof(float), 256));
  a.chunk_tab = (int32_t*)((char*)a.seq_order + align_up((size_t)batch * sizeof(int32_t), 256));
  a.unit_tab = (int32_t*)((char*)a.chunk_tab + align_up((size_t)batch * sizeof(int32_t), 256));
  a.balanced = false;
  a.rows_bf16 = false;
  a.q_group = q_group;
  a.latent = c->latent;
  a.rope = c->rope;
  a.page_table = c->page_table;
  a.seq_lens = c->seq_lens;
  a.page_size = c->page_size;
  a.max_pages = c->max_pages_per_seq;
  a.n_blocks = c->n_blocks;
  a.d_cb = c->d_cb;
  a.d_r = c->d_r;
  a.batch = batch;
  a.h = h;
  a.groups = groups;
  a.d_h = d_h;
  a.q_abs = q_abs;
  a.q_rope = q_rope;
  a.w_uv = w_uv;
  a.softmax_scale = softmax_scale;
  a.out_scale = out_scale;
  a.out = out;
  a.out_dtype = out_dtype;
  a.lse = lse;
  a.gate = gate;
  a.dtype = c->dtype;
  a.stream = (hipStream_t)stream;
  a.t_main = timing_pair(0);
  a.t_epi = timing_pair(1);
  // chunk lengths that follow the sequence lengths need both MFMA kernels (they read the table)
  if (a.plan.target_chunks > 0 && merge_upproj_mfma_supported(a) &&
      (decode_mfma_supported(a) || decode_gla_supported(a) || mla_mfma_supported(a)))
    a.balanced = launch_plan_chunks(a) == MLRA_OK;
  // the MLRA MFMA kernels hand the epilogue normalised bf16 rows (one per chunk) instead of fp32 partials
  a.rows_bf16 = merge_upproj_mfma_supported(a) && (decode_mfma_supported(a) || decode_gla_supported(a));
  // the MFMA launchers record their kernel's own start and end; the generic kernels are bracketed by stream markers
  const bool main_fast = decode_mfma_supported(a) || decode_gla_supported(a) || mla_mfma_supported(a);
  const bool epi_fast = merge_upproj_mfma_supported(a);
  if (a.t_main.on() && !main_fast) (void)hipEventRecord(a.t_main.start, a.stream);
  int st = decode_mfma_supported(a) ? launch_decode_mfma(a)
           : decode_gla_supported(a) ? launch_decode_gla(a)
           : mla_mfma_supported(a)  ? launch_mla_mfma(a)
                                    : launch_decode_generic(a);
  if (st != MLRA_OK) return st;
  if (a.t_main.on() && !main_fast) (void)hipEventRecord(a.t_main.stop, a.stream);
  if (a.t_epi.on() && !epi_fast) (void)hipEventRecord(a.t_epi.start, a.stream);
  st = epi_fast ? launch_merge_upproj_mfma(a) : launch_merge_upproj_generic(a);
  if (a.t_epi.on() && !epi_fast) (void)hipEventRecord(a.t_epi.stop, a.stream);
  if (st == MLRA_OK && timing_on()) ++g_timing_calls;
  return st;
}

}  // namespace mlra

using namespace mlra;

extern "C" {

const char* mlra_strerror(int status) {
  switch (status) {
    case MLRA_OK: return "ok";
    case MLRA_ERR_NULL: return "a required pointer is NULL";
    case MLRA_ERR_SHAPE: return "a dimension is non-positive or not supported";
    case MLRA_ERR_DTYPE: return "unknown or unsupported element type";
    case MLRA_ERR_WORKSPACE: return "workspace missing, misaligned or smaller than required";
    case MLRA_ERR_LAUNCH: return "the HIP runtime refused a launch or a query";
    default: return "unknown status";
  }
}

int mlra_append_kv(const mlra_cache* c, int32_t batch, const void* c_kv_new, const void* k_rope_new,
                   int32_t src_dtype, const int32_t* positions, void* stream) {
  if (!c || !c_kv_new || !k_rope_new || !positions) return MLRA_ERR_NULL;
  if (!c->latent || !c->rope || !c->page_table) return MLRA_ERR_NULL;
  if (!valid_dtype(c->dtype) || !valid_dtype(src_dtype)) return MLRA_ERR_DTYPE;
  if (batch <= 0 || c->n_blocks <= 0 || c->d_cb <= 0 || c->d_r <= 0 || c->page_size <= 0 ||
      c->max_pages_per_seq <= 0 || c->num_pages <= 0)
    return MLRA_ERR_SHAPE;
  return launch_append_kv(c, batch, c_kv_new, k_rope_new, src_dtype, positions, (hipStream_t)stream);
}

static int absorb_common(int batch, int h, int d_h, int n_blocks, int groups, int d_cb, int d_r, const void* q_nope,
                         const void* w_uk, const void* q_rope, float fold, void* q_abs, void* q_rope_out, int dtype,
                         void* stream) {
  if (!q_nope || !w_uk || !q_abs) return MLRA_ERR_NULL;
  if (!valid_dtype(dtype)) return MLRA_ERR_DTYPE;
  if (batch <= 0 || h <= 0 || d_h <= 0 || n_blocks <= 0 || d_cb <= 0) return MLRA_ERR_SHAPE;
  if (h % groups != 0 || n_blocks % groups != 0) return MLRA_ERR_SHAPE;
  if (h > 65535 || batch > 65535 || n_blocks > 65534 || d_h > 8192) return MLRA_ERR_SHAPE;
  if (absorb_q_mfma_supported(d_h, d_cb, dtype) && (!q_rope_out || d_r % 8 == 0))
    return launch_absorb_q_mfma(batch, h / groups, d_h, n_blocks, groups, d_cb, q_nope, w_uk, q_abs,
                                (hipStream_t)stream, fold, q_rope, q_rope_out, d_r);
  return launch_absorb_q_generic(batch, h / groups, d_h, n_blocks, groups, d_cb, q_nope, w_uk, q_abs, dtype,
                                 (hipStream_t)stream, fold, q_rope, q_rope_out, d_r);
}

static int absorb_folded(int batch, int h, int d_h, int n_blocks, int groups, int d_cb, int d_r, const void* q_nope,
                         const void* w_uk, const void* q_rope, float softmax_scale, void* q_abs, void* q_rope_out,
                         int dtype, void* stream) {
  if (!q_rope || !q_rope_out) return MLRA_ERR_NULL;
  if (!(softmax_scale > 0.f) || d_r <= 0) return MLRA_ERR_SHAPE;
  return absorb_common(batch, h, d_h, n_blocks, groups, d_cb, d_r, q_nope, w_uk, q_rope,
                       softmax_scale * 1.4426950408889634f, q_abs, q_rope_out, dtype, stream);
}

int mlra_absorb_q(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb, const void* q_nope,
                  const void* w_uk, void* q_abs, int32_t dtype, void* stream) {
  return absorb_common(batch, h, d_h, n_blocks, 1, d_cb, 0, q_nope, w_uk, nullptr, 1.f, q_abs, nullptr, dtype, stream);
}

int mlra_absorb_q_folded(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb, int32_t d_r,
                         const void* q_nope, const void* w_uk, const void* q_rope, float softmax_scale, void* q_abs,
                         void* q_rope_out, int32_t dtype, void* stream) {
  return absorb_folded(batch, h, d_h, n_blocks, 1, d_cb, d_r, q_nope, w_uk, q_rope, softmax_scale, q_abs, q_rope_out,
                       dtype, stream);
}

size_t mlra_decode_workspace_bytes(int32_t batch, int32_t h, int32_t n_blocks, int32_t d_cb, int32_t max_seq_len) {
  if (batch <= 0 || h <= 0 || n_blocks <= 0 || d_cb <= 0 || max_seq_len <= 0) return 0;
  return decode_ws_bytes(batch, h, n_blocks, d_cb, plan_decode(batch, h, n_blocks, d_cb, max_seq_len));
}

int mlra_decode_attn(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                     const void* q_rope, const void* w_uv, float softmax_scale, float out_scale, void* out,
                     int32_t out_dtype, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_common(cache, batch, h, 1, d_h, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype, lse,
                       workspace, workspace_bytes, stream);
}

int mlra_decode_attn_static(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                            const void* q_rope, const void* w_uv, float softmax_scale, float out_scale, void* out,
                            int32_t out_dtype, float* lse, void* stream) {
  if (!cache) return MLRA_ERR_NULL;
  if (batch <= 0 || h <= 0 || cache->n_blocks <= 0 || cache->d_cb <= 0 || cache->page_size <= 0 ||
      cache->max_pages_per_seq <= 0 || (long)cache->max_pages_per_seq * cache->page_size > 0x7fffffffL)
    return MLRA_ERR_SHAPE;
  const size_t need = mlra_decode_workspace_bytes(batch, h, cache->n_blocks, cache->d_cb,
                                                  cache->max_pages_per_seq * cache->page_size);
  if (need == 0) return MLRA_ERR_SHAPE;
  if (need > kStaticScratchBytes) return MLRA_ERR_WORKSPACE;   // beyond the built-in scratch: use mlra_decode_attn
  void* ptr = nullptr;
  const int st = static_scratch(&ptr);
  if (st != MLRA_OK) return st;
  // (every partial, table and row that the kernels read from the scratch is written earlier in the same
  // call, so what the previous call left there is never read and nothing needs clearing)
  return decode_common(cache, batch, h, 1, d_h, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype, lse,
                       ptr, kStaticScratchBytes, stream);
}

size_t mlra_decode_multi_workspace_bytes(int32_t batch, int32_t q_len, int32_t h, int32_t n_blocks, int32_t d_cb,
                                         int32_t page_size, int32_t max_pages_per_seq) {
  if (batch <= 0 || q_len <= 0 || h <= 0 || n_blocks <= 0 || d_cb <= 0 || page_size <= 0 || max_pages_per_seq <= 0)
    return 0;
  if ((long)batch * q_len > 65535 || (long)max_pages_per_seq * page_size > 0x7fffffffL) return 0;
  const int units = batch * q_len;
  return align_up((size_t)units * sizeof(int32_t), 256) +
         align_up((size_t)units * max_pages_per_seq * sizeof(int32_t), 256) +
         mlra_decode_workspace_bytes(units, h, n_blocks, d_cb, max_pages_per_seq * page_size);
}

int mlra_decode_attn_multi(const mlra_cache* c, int32_t batch, int32_t q_len, int32_t h, int32_t d_h,
                           const void* q_abs, const void* q_rope, const void* w_uv, float softmax_scale,
                           float out_scale, void* out, int32_t out_dtype, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (!c || !c->page_table || !c->seq_lens) return MLRA_ERR_NULL;
  if (batch <= 0 || q_len <= 0 || (long)batch * q_len > 65535 || c->max_pages_per_seq <= 0 || c->page_size <= 0)
    return MLRA_ERR_SHAPE;
  if (q_len == 1)
    return decode_common(c, batch, h, 1, d_h, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype, lse,
                         workspace, workspace_bytes, stream);
  const int units = batch * q_len;
  const size_t lens_bytes = align_up((size_t)units * sizeof(int32_t), 256);
  const size_t table_bytes = align_up((size_t)units * c->max_pages_per_seq * sizeof(int32_t), 256);
  if (!workspace || ((uintptr_t)workspace) % 256 != 0 || workspace_bytes < lens_bytes + table_bytes)
    return MLRA_ERR_WORKSPACE;
  // every host-checkable condition of the decode proper is checked here first, so that an error return
  // never leaves the expansion kernel enqueued
  const size_t need = mlra_decode_multi_workspace_bytes(batch, q_len, h, c->n_blocks, c->d_cb, c->page_size,
                                                        c->max_pages_per_seq);
  if (need == 0) return MLRA_ERR_SHAPE;
  if (workspace_bytes < need) return MLRA_ERR_WORKSPACE;
  if (!q_abs || !q_rope || !w_uv || !out || !c->latent || !c->rope) return MLRA_ERR_NULL;
  if (!valid_dtype(c->dtype) || !valid_dtype(out_dtype)) return MLRA_ERR_DTYPE;
  if (h <= 0 || d_h <= 0 || c->n_blocks <= 0 || c->d_cb <= 0 || c->d_r <= 0 || c->num_pages <= 0) return MLRA_ERR_SHAPE;
  int32_t* lens2 = (int32_t*)workspace;
  int32_t* table2 = (int32_t*)((char*)workspace + lens_bytes);
  int st = launch_expand_queries(c->seq_lens, c->page_table, batch, q_len, c->max_pages_per_seq, lens2, table2,
                                 (hipStream_t)stream);
  if (st != MLRA_OK) return st;
  mlra_cache c2 = *c;
  c2.page_table = table2;
  c2.seq_lens = lens2;
  return decode_common(&c2, units, h, 1, d_h, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype, lse,
                       (char*)workspace + lens_bytes + table_bytes, workspace_bytes - lens_bytes - table_bytes,
                       stream, nullptr, q_len);
}

int mlra_decode_attn_gated(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                           const void* q_rope, const void* w_uv, const void* gate, float softmax_scale,
                           float out_scale, void* out, int32_t out_dtype, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (!gate) return MLRA_ERR_NULL;
  return decode_common(cache, batch, h, 1, d_h, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype, lse,
                       workspace, workspace_bytes, stream, gate);
}

int mlra2_absorb_q(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb, const void* q_nope,
                   const void* w_uk, void* q_abs, int32_t dtype, void* stream) {
  if (h % 2 != 0 || n_blocks % 2 != 0) return (!q_nope || !w_uk || !q_abs) ? MLRA_ERR_NULL : MLRA_ERR_SHAPE;
  return absorb_common(batch, h, d_h, n_blocks, 2, d_cb, 0, q_nope, w_uk, nullptr, 1.f, q_abs, nullptr, dtype, stream);
}

int mlra2_absorb_q_folded(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb, int32_t d_r,
                          const void* q_nope, const void* w_uk, const void* q_rope, float softmax_scale, void* q_abs,
                          void* q_rope_out, int32_t dtype, void* stream) {
  if (h % 2 != 0 || n_blocks % 2 != 0) return (!q_nope || !w_uk || !q_abs) ? MLRA_ERR_NULL : MLRA_ERR_SHAPE;
  return absorb_folded(batch, h, d_h, n_blocks, 2, d_cb, d_r, q_nope, w_uk, q_rope, softmax_scale, q_abs, q_rope_out,
                       dtype, stream);
}

size_t mlra2_decode_workspace_bytes(int32_t batch, int32_t h, int32_t n_blocks, int32_t d_cb, int32_t max_seq_len) {
  if (batch <= 0 || h <= 0 || n_blocks <= 0 || d_cb <= 0 || max_seq_len <= 0) return 0;
  if (h % 2 != 0 || n_blocks % 2 != 0) return 0;
  return decode_ws_bytes(batch, h / 2, n_blocks, d_cb, plan_decode(batch, h / 2, n_blocks, d_cb, max_seq_len));
}

int mlra2_decode_attn(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                      const void* q_rope, const void* w_uv, float softmax_scale, float out_scale, void* out,
                      int32_t out_dtype, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  if (h <= 0 || h % 2 != 0) return MLRA_ERR_SHAPE;
  if (cache && cache->n_blocks % 2 != 0) return MLRA_ERR_SHAPE;
  return decode_common(cache, batch, h / 2, 2, d_h, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype,
                       lse, workspace, workspace_bytes, stream);
}

size_t mlra_pre_attention_workspace_bytes(int32_t batch, int32_t d, int32_t d_cq, int32_t n_blocks, int32_t d_cb,
                                          int32_t d_r, int32_t h, int32_t d_h, int32_t dtype) {
  if (batch <= 0 || d <= 0 || d_cq <= 0 || n_blocks <= 0 || d_cb <= 0 || d_r <= 0 || h <= 0 || d_h <= 0) return 0;
  if (!valid_dtype(dtype) || d_r % 2 != 0 || d_h % 2 != 0 || d_r > 256) return 0;
  return pre_plan(dtype, batch, d, d_cq, n_blocks * d_cb, d_r, h, d_h).bytes;
}

int mlra_pre_attention(const mlra_cache* c, const mlra_pre_weights* w, int32_t batch, const void* hidden,
                       const int32_t* positions, void* q_nope, void* q_rope, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (!c || !w || !hidden || !positions || !q_nope || !q_rope) return MLRA_ERR_NULL;
  if (!c->latent || !c->rope || !c->page_table) return MLRA_ERR_NULL;
  if (!w->w_dq || !w->w_dkv || !w->w_kr || !w->w_uq || !w->w_qr) return MLRA_ERR_NULL;
  if (!valid_dtype(c->dtype) || !valid_dtype(w->dtype)) return MLRA_ERR_DTYPE;
  if (batch <= 0 || batch > 65535 || w->d <= 0 || w->d_cq <= 0 || w->h <= 0 || w->d_h <= 0 || c->n_blocks <= 0 ||
      c->d_cb <= 0 || c->d_r <= 0 || c->page_size <= 0 || c->max_pages_per_seq <= 0 || c->num_pages <= 0)
    return MLRA_ERR_SHAPE;
  if (c->d_r % 2 != 0 || w->d_h % 2 != 0 || c->d_r > 256) return MLRA_ERR_SHAPE;
  if ((long)w->h * (w->d_h + c->d_r) > (1L << 24) || (long)w->d_cq + (long)c->n_blocks * c->d_cb > 12000)
    return MLRA_ERR_SHAPE;
  const size_t need = mlra_pre_attention_workspace_bytes(batch, w->d, w->d_cq, c->n_blocks, c->d_cb, c->d_r, w->h,
                                                         w->d_h, w->dtype);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace) % 256 != 0) return MLRA_ERR_WORKSPACE;
  return launch_pre_attention(c, w, batch, hidden, positions, q_nope, q_rope, workspace, (hipStream_t)stream);
}

int mla_decode_attn(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                    const void* q_rope, const void* w_uv, float softmax_scale, void* out, int32_t out_dtype,
                    float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  if (cache && cache->n_blocks != 1) return MLRA_ERR_SHAPE;
  return decode_common(cache, batch, h, 1, d_h, q_abs, q_rope, w_uv, softmax_scale, 1.0f, out, out_dtype, lse,
                       workspace, workspace_bytes, stream);
}

int mlra_decode_plan_info(int32_t batch, int32_t h, int32_t d_h, int32_t groups, int32_t n_blocks, int32_t d_cb,
                          int32_t d_r, int32_t page_size, int32_t max_seq_len, int32_t dtype, int32_t* info) {
  if (!info) return MLRA_ERR_NULL;
  if (!valid_dtype(dtype)) return MLRA_ERR_DTYPE;
  if (batch <= 0 || h <= 0 || d_h <= 0 || groups <= 0 || n_blocks <= 0 || d_cb <= 0 || d_r <= 0 || page_size <= 0 ||
      max_seq_len <= 0 || h % groups != 0 || n_blocks % groups != 0)
    return MLRA_ERR_SHAPE;
  DecodeArgs a = {};
  a.batch = batch;
  a.h = h / groups;          // heads served by one block
  a.groups = groups;
  a.d_h = d_h;
  a.n_blocks = n_blocks;
  a.d_cb = d_cb;
  a.d_r = d_r;
  a.page_size = page_size;
  a.max_pages = (max_seq_len + page_size - 1) / page_size;
  a.dtype = dtype;
  a.plan = plan_decode(batch, a.h, n_blocks, d_cb, a.max_pages * page_size);
  info[0] = decode_mfma_supported(a) ? (decode_mfma_paired(a.h, n_blocks) ? 2 : 1)
            : decode_gla_supported(a) ? 3
            : mla_mfma_supported(a)  ? 4
                                     : 0;
  info[1] = a.plan.n_splits;
  info[2] = a.plan.chunk_tokens;
  info[3] = a.plan.target_chunks;
  info[4] = a.plan.single_if_uniform ? 1 : 0;
  info[5] = merge_upproj_mfma_supported(a) ? 1 : 0;
  return MLRA_OK;
}

int mlra_kernel_timing_begin(int32_t max_calls) {
  if (max_calls <= 0 || max_calls > 100000) return MLRA_ERR_SHAPE;
  for (hipEvent_t e : g_events) (void)hipEventDestroy(e);
  g_events.assign((size_t)4 * max_calls, nullptr);
  for (hipEvent_t& e : g_events)
    if (hipEventCreate(&e) != hipSuccess) return MLRA_ERR_LAUNCH;
  g_timing_calls = 0;
  g_timing_cap = max_calls;
  return MLRA_OK;
}

int mlra_kernel_timing_end(double* main_kernel_ms, double* epilogue_kernel_ms, int32_t* calls) {
  if (!main_kernel_ms || !epilogue_kernel_ms || !calls) return MLRA_ERR_NULL;
  double a = 0.0, b = 0.0;
  int st = MLRA_OK;
  for (int i = 0; i < g_timing_calls; ++i) {
    float ms0 = 0.f, ms1 = 0.f;
    if (hipEventSynchronize(g_events[4 * i + 3]) != hipSuccess ||
        hipEventElapsedTime(&ms0, g_events[4 * i], g_events[4 * i + 1]) != hipSuccess ||
        hipEventElapsedTime(&ms1, g_events[4 * i + 2], g_events[4 * i + 3]) != hipSuccess) {
      st = MLRA_ERR_LAUNCH;
      break;
    }
    a += ms0;
    b += ms1;
  }
  *calls = g_timing_calls;
  *main_kernel_ms = g_timing_calls ? a / g_timing_calls : 0.0;
  *epilogue_kernel_ms = g_timing_calls ? b / g_timing_calls : 0.0;
  for (hipEvent_t e : g_events) (void)hipEventDestroy(e);
  g_events.clear();
  g_timing_cap = g_timing_calls = 0;
  return st;
}

size_t gqa_decode_workspace_bytes(int32_t batch, int32_t h, int32_t d_h, int32_t max_seq_len) {
  if (batch <= 0 || h <= 0 || d_h <= 0 || max_seq_len <= 0) return 0;
  const SplitPlan p = plan_splits(batch, 1, max_seq_len);
  const size_t units = (size_t)batch * p.n_splits;
  return align_up(units * h * d_h * sizeof(float), 256) + align_up(units * h * 2 * sizeof(float), 256);
}

int gqa_decode_attn(const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_lens,
                    int32_t num_pages, int32_t page_size, int32_t max_pages_per_seq, int32_t batch, int32_t h,
                    int32_t g, int32_t d_h, int32_t dtype, const void* q, float softmax_scale, void* out,
                    int32_t out_dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (!k_pool || !v_pool || !page_table || !seq_lens || !q || !out) return MLRA_ERR_NULL;
  if (!valid_dtype(dtype) || !valid_dtype(out_dtype)) return MLRA_ERR_DTYPE;
  if (num_pages <= 0 || page_size <= 0 || max_pages_per_seq <= 0 || batch <= 0 || h <= 0 || g <= 0 || d_h <= 0)
    return MLRA_ERR_SHAPE;
  if (h % g != 0 || h > 65535 || batch > 65535 || d_h > 1024) return MLRA_ERR_SHAPE;
  if ((long)max_pages_per_seq * page_size > 0x7fffffffL) return MLRA_ERR_SHAPE;
  GqaArgs a;
  a.page_size = page_size;
  a.h = h;
  a.g = g;
  a.d_h = d_h;
  a.dtype = dtype;
  // the MFMA kernel runs one workgroup per (sequence, KV head, chunk), the generic one splits further
  a.plan = plan_splits(batch, g, max_pages_per_seq * page_size);
  const bool use_mfma = gqa_mfma_supported(a);
  if (!use_mfma) a.plan = plan_splits(batch, 1, max_pages_per_seq * page_size);
  const size_t units = (size_t)batch * a.plan.n_splits;
  const size_t need = align_up(units * h * d_h * sizeof(float), 256) + align_up(units * h * 2 * sizeof(float), 256);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace) % 256 != 0) return MLRA_ERR_WORKSPACE;
  a.part_o = (float*)workspace;
  a.part_ml = (float*)((char*)workspace + align_up(units * h * d_h * sizeof(float), 256));
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.page_table = page_table;
  a.seq_lens = seq_lens;
  a.page_size = page_size;
  a.max_pages = max_pages_per_seq;
  a.batch = batch;
  a.h = h;
  a.g = g;
  a.d_h = d_h;
  a.dtype = dtype;
  a.q = q;
  a.softmax_scale = softmax_scale;
  a.out = out;
  a.out_dtype = out_dtype;
  a.stream = (hipStream_t)stream;
  int st = use_mfma ? launch_gqa_mfma(a) : launch_gqa_generic(a);
  if (st != MLRA_OK) return st;
  return launch_gqa_merge(a);
}

}  // extern "C"
