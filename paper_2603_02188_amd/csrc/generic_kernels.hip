// Shape-generic kernels of libmlra: cache append, query absorption, a plain (non-MFMA) decode
// kernel for any dims and for fp32 caches, and the split merge + up-projection epilogue.
// All arithmetic is fp32; bf16 appears only as a storage type.
#include "mlra_internal.h"

namespace mlra {

static constexpr float kLog2e = 1.4426950408889634f;
static constexpr float kLn2 = 0.6931471805599453f;
static constexpr float kNegBig = -1.0e30f;  // "no token seen yet" running max (finite: no inf-inf)

__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ------------------------------------------------------------------------------------------------
// mlra_append_kv: one workgroup per sequence stores the newest row (Section 2.1: C^KV and K^RoPE of
// every token are cached).
// ------------------------------------------------------------------------------------------------
template <typename TC, typename TS>
__global__ void append_kv_kernel(TC* latent, TC* rope, const int32_t* page_table, const int32_t* positions,
                                 const TS* c_kv_new, const TS* k_rope_new, int page_size, int max_pages,
                                 int n_blocks, int d_cb, int d_r) {
  const int s = blockIdx.x;
  const int pos = positions[s];
  if (pos < 0) return;
  const int page = page_table[(size_t)s * max_pages + pos / page_size];
  const int slot = pos % page_size;
  const int d_c = n_blocks * d_cb;
  for (int e = threadIdx.x; e < d_c + d_r; e += blockDim.x) {
    if (e < d_c) {
      const int b = e / d_cb, c = e % d_cb;
      const size_t dst = (((size_t)page * n_blocks + b) * page_size + slot) * d_cb + c;
      store_f32(latent, dst, load_f32(c_kv_new, (size_t)s * d_c + e));
    } else {
      const int c = e - d_c;
      const size_t dst = ((size_t)page * page_size + slot) * d_r + c;
      store_f32(rope, dst, load_f32(k_rope_new, (size_t)s * d_r + c));
    }
  }
}

int launch_append_kv(const mlra_cache* c, int batch, const void* c_kv_new, const void* k_rope_new, int src_dtype,
                     const int32_t* positions, hipStream_t stream) {
#define MLRA_APPEND(TC, TS)                                                                                     \
  append_kv_kernel<TC, TS><<<batch, 256, 0, stream>>>((TC*)c->latent, (TC*)c->rope, c->page_table, positions,   \
                                                      (const TS*)c_kv_new, (const TS*)k_rope_new, c->page_size, \
                                                      c->max_pages_per_seq, c->n_blocks, c->d_cb, c->d_r)
  if (c->dtype == MLRA_BF16 && src_dtype == MLRA_F32) MLRA_APPEND(bf16_t, float);
  else if (c->dtype == MLRA_BF16 && src_dtype == MLRA_BF16) MLRA_APPEND(bf16_t, bf16_t);
  else if (c->dtype == MLRA_F32 && src_dtype == MLRA_F32) MLRA_APPEND(float, float);
  else MLRA_APPEND(float, bf16_t);
#undef MLRA_APPEND
  return check_launch();
}

// ------------------------------------------------------------------------------------------------
// Several query tokens per sequence: every (sequence, query) pair becomes a decode unit of its own with
// the sequence's pages and the length of the query's causal prefix.
// ------------------------------------------------------------------------------------------------
__global__ void expand_queries_kernel(const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ page_table,
                                      int q_len, int max_pages, int32_t* __restrict__ seq_lens_out,
                                      int32_t* __restrict__ page_table_out) {
  const int u = blockIdx.x, s = u / q_len, j = u % q_len;
  if (threadIdx.x == 0) seq_lens_out[u] = max(0, seq_lens[s] - (q_len - 1 - j));
  for (int p = threadIdx.x; p < max_pages; p += blockDim.x)
    page_table_out[(size_t)u * max_pages + p] = page_table[(size_t)s * max_pages + p];
}

int launch_expand_queries(const int32_t* seq_lens, const int32_t* page_table, int batch, int q_len, int max_pages,
                          int32_t* seq_lens_out, int32_t* page_table_out, hipStream_t stream) {
  expand_queries_kernel<<<batch * q_len, 256, 0, stream>>>(seq_lens, page_table, q_len, max_pages, seq_lens_out,
                                                           page_table_out);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------
// mlra_absorb_q, generic form (Step 1, Section 2.1): one workgroup per (head, block, sequence);
// each wave produces rows c of q~ = W^UK_(b),(i) q with lanes striding the d_h contraction.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void absorb_q_generic_kernel(const T* q_nope, const T* w_uk, T* q_abs, int h, int d_h, int n_blocks,
                                        int groups, int d_cb, float fold, const T* q_rope, T* q_rope_out, int d_r) {
  extern __shared__ float qs[];
  const int head = blockIdx.x, b = blockIdx.y, s = blockIdx.z;
  if (b == n_blocks) {   // (launched only when the softmax scale is folded in) the RoPE queries of this head
    for (int id = threadIdx.x; id < groups * d_r; id += blockDim.x) {
      const size_t off = ((size_t)s * h * groups + (id / d_r) * h + head) * d_r + id % d_r;
      store_f32(q_rope_out, off, load_f32(q_rope, off) * fold);
    }
    return;
  }
  const int q_head = (b / (n_blocks / groups)) * h + head;   // Eq. (6): block b serves the heads of its group
  for (int p = threadIdx.x; p < d_h; p += blockDim.x)
    qs[p] = load_f32(q_nope, ((size_t)s * h * groups + q_head) * d_h + p);
  __syncthreads();
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, nwaves = blockDim.x / 64;
  for (int c = wave; c < d_cb; c += nwaves) {
    const size_t row = ((size_t)b * d_cb + c) * ((size_t)h * d_h) + (size_t)head * d_h;
    float acc = 0.f;
    for (int p = lane; p < d_h; p += 64) acc += load_f32(w_uk, row + p) * qs[p];
    acc = wave_sum(acc);
    if (lane == 0) store_f32(q_abs, (((size_t)s * n_blocks + b) * h + head) * d_cb + c, acc * fold);
  }
}

int launch_absorb_q_generic(int batch, int h, int d_h, int n_blocks, int groups, int d_cb, const void* q_nope,
                            const void* w_uk, void* q_abs, int dtype, hipStream_t stream, float fold,
                            const void* q_rope, void* q_rope_out, int d_r) {
  dim3 grid(h, n_blocks + (q_rope_out ? 1 : 0), batch);
  const size_t lds = (size_t)d_h * sizeof(float);
  if (dtype == MLRA_BF16)
    absorb_q_generic_kernel<bf16_t><<<grid, 256, lds, stream>>>((const bf16_t*)q_nope, (const bf16_t*)w_uk,
                                                                (bf16_t*)q_abs, h, d_h, n_blocks, groups, d_cb, fold,
                                                                (const bf16_t*)q_rope, (bf16_t*)q_rope_out, d_r);
  else
    absorb_q_generic_kernel<float><<<grid, 256, lds, stream>>>((const float*)q_nope, (const float*)w_uk,
                                                               (float*)q_abs, h, d_h, n_blocks, groups, d_cb, fold,
                                                               (const float*)q_rope, (float*)q_rope_out, d_r);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------
// Generic decode (Step 2 per block, Eq. (1)): one workgroup per (context chunk, block x head group,
// sequence).  A tile of TT tokens [C_b | K^RoPE] sits in LDS as fp32 and serves as key and value.
// Partials are written unnormalised with the running max m and sum l in the log2 domain:
//   m = max_t score_t * log2(e),  l = sum_t 2^(score_t*log2(e) - m),  z = sum_t 2^(...) C_b[t].
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void decode_generic_kernel(
    const T* __restrict__ latent, const T* __restrict__ rope, const int32_t* __restrict__ page_table,
    const int32_t* __restrict__ seq_lens, int page_size, int max_pages, int n_blocks, int d_cb, int d_r, int h,
    const T* __restrict__ q_abs, const T* __restrict__ q_rope, float scale_log2, float* __restrict__ part_z,
    float* __restrict__ part_ml, int n_splits, int chunk, int HG, int TT, int groups) {
  extern __shared__ float smem[];
  const int D = d_cb + d_r, DP = D + 1;
  float* qs = smem;                 // [HG][D]
  float* tile = qs + HG * D;        // [TT][DP]
  float* ps = tile + TT * DP;       // [HG][TT]
  float* zs = ps + HG * TT;         // [HG][d_cb]
  float* ms = zs + HG * d_cb;       // [HG]
  float* ls = ms + HG;              // [HG]
  float* al = ls + HG;              // [HG]

  const int split = blockIdx.x;
  const int n_hg = (h + HG - 1) / HG;
  const int b = blockIdx.y / n_hg, hg = blockIdx.y % n_hg;
  const int s = blockIdx.z;
  const int n = seq_lens[s];
  const int t0 = split * chunk;
  if (t0 >= n) return;
  const int t1 = min(n, t0 + chunk);
  const int head0 = hg * HG;
  const int nh = min(HG, h - head0);
  const int tid = threadIdx.x;
  const int rope_head0 = (b / (n_blocks / groups)) * h;   // first head of this block's group in q_rope

  for (int idx = tid; idx < nh * D; idx += 256) {
    const int hh = idx / D, k = idx % D;
    const int head = head0 + hh;
    qs[hh * D + k] = k < d_cb ? load_f32(q_abs, (((size_t)s * n_blocks + b) * h + head) * d_cb + k)
                              : load_f32(q_rope, ((size_t)s * h * groups + rope_head0 + head) * d_r + (k - d_cb));
  }
  for (int idx = tid; idx < HG * d_cb; idx += 256) zs[idx] = 0.f;
  if (tid < HG) { ms[tid] = kNegBig; ls[tid] = 0.f; al[tid] = 1.f; }
  __syncthreads();

  for (int tb = t0; tb < t1; tb += TT) {
    // tile load: rows beyond the chunk are zero-filled so that 0-weight rows stay finite
    for (int idx = tid; idx < TT * D; idx += 256) {
      const int t = idx / D, k = idx % D;
      const int tok = tb + t;
      float v = 0.f;
      if (tok < t1) {
        const int page = page_table[(size_t)s * max_pages + tok / page_size];
        const int slot = tok % page_size;
        v = k < d_cb ? load_f32(latent, (((size_t)page * n_blocks + b) * page_size + slot) * d_cb + k)
                     : load_f32(rope, ((size_t)page * page_size + slot) * d_r + (k - d_cb));
      }
      tile[t * DP + k] = v;
    }
    __syncthreads();
    for (int idx = tid; idx < nh * TT; idx += 256) {
      const int hh = idx / TT, t = idx % TT;
      float acc = 0.f;
      const float* q = qs + hh * D;
      const float* kr = tile + t * DP;
      for (int k = 0; k < D; ++k) acc += q[k] * kr[k];
      ps[hh * TT + t] = (tb + t < t1) ? acc * scale_log2 : -INFINITY;
    }
    __syncthreads();
    {
      const int wave = tid / 64, lane = tid % 64;
      for (int hh = wave; hh < nh; hh += 4) {
        const float sc = lane < TT ? ps[hh * TT + lane] : -INFINITY;
        const float m_old = ms[hh];
        const float m_new = fmaxf(m_old, wave_max(sc));
        const float p = exp2f(sc - m_new);  // masked rows: 2^(-inf) = 0
        const float sum = wave_sum(p);
        if (lane < TT) ps[hh * TT + lane] = p;
        if (lane == 0) {
          const float a = exp2f(m_old - m_new);
          al[hh] = a;
          ms[hh] = m_new;
          ls[hh] = ls[hh] * a + sum;
        }
      }
    }
    __syncthreads();
    for (int idx = tid; idx < nh * d_cb; idx += 256) {
      const int hh = idx / d_cb, c = idx % d_cb;
      float acc = zs[idx] * al[hh];
      const float* p = ps + hh * TT;
      for (int t = 0; t < TT; ++t) acc += p[t] * tile[t * DP + c];
      zs[idx] = acc;
    }
    __syncthreads();
  }

  const size_t unit = ((size_t)s * n_blocks + b) * n_splits + split;
  for (int idx = tid; idx < nh * d_cb; idx += 256) {
    const int hh = idx / d_cb, c = idx % d_cb;
    part_z[(unit * h + head0 + hh) * d_cb + c] = zs[idx];
  }
  if (tid < nh) {
    part_ml[(unit * h + head0 + tid) * 2 + 0] = ms[tid];
    part_ml[(unit * h + head0 + tid) * 2 + 1] = ls[tid];
  }
}

int launch_decode_generic(const DecodeArgs& a) {
  const int D = a.d_cb + a.d_r;
  const int HG = 8;
  int TT = 64;
  auto lds_bytes = [&](int tt) { return (size_t)(HG * D + tt * (D + 1) + HG * tt + HG * a.d_cb + 3 * HG) * 4; };
  while (TT > 1 && lds_bytes(TT) > 64 * 1024) TT >>= 1;
  if (lds_bytes(TT) > 64 * 1024) return MLRA_ERR_SHAPE;
  const int n_hg = (a.h + HG - 1) / HG;
  dim3 grid(a.plan.n_splits, a.n_blocks * n_hg, a.batch);
  const float scale_log2 = softmax_scale_log2(a.softmax_scale);
  if (a.dtype == MLRA_BF16)
    decode_generic_kernel<bf16_t><<<grid, 256, lds_bytes(TT), a.stream>>>(
        (const bf16_t*)a.latent, (const bf16_t*)a.rope, a.page_table, a.seq_lens, a.page_size, a.max_pages,
        a.n_blocks, a.d_cb, a.d_r, a.h, (const bf16_t*)a.q_abs, (const bf16_t*)a.q_rope, scale_log2, a.part_z,
        a.part_ml, a.plan.n_splits, a.plan.chunk_tokens, HG, TT, a.groups);
  else
    decode_generic_kernel<float><<<grid, 256, lds_bytes(TT), a.stream>>>(
        (const float*)a.latent, (const float*)a.rope, a.page_table, a.seq_lens, a.page_size, a.max_pages,
        a.n_blocks, a.d_cb, a.d_r, a.h, (const float*)a.q_abs, (const float*)a.q_rope, scale_log2, a.part_z,
        a.part_ml, a.plan.n_splits, a.plan.chunk_tokens, HG, TT, a.groups);
  return check_launch();
}

// ------------------------------------------------------------------------------------------------
// Split merge + Step 3 + block sum, generic form: one workgroup per (head, sequence).
//   z_b = sum_s 2^(m_s - m*) z_s / sum_s 2^(m_s - m*) l_s        (log-sum-exp merge of the chunks)
//   out = out_scale * sum_b z_b W^UV_(b),(i)                       (Step 3 and Eq. (5)'s block sum)
// ------------------------------------------------------------------------------------------------
template <typename T, typename TO>
__global__ __launch_bounds__(256) void merge_upproj_generic_kernel(
    const float* __restrict__ part_z, const float* __restrict__ part_ml, const int32_t* __restrict__ seq_lens,
    const T* __restrict__ w_uv, TO* __restrict__ out, float* __restrict__ lse, int h, int d_h, int n_blocks,
    int d_cb, int n_splits, int chunk, float out_scale, int groups, const T* __restrict__ gate) {
  extern __shared__ float zs[];  // [bpg*d_cb]
  // output head blockIdx.x = grp * h + head; its branches are the bpg blocks of group grp (Eq. (6);
  // one group of all blocks is Eq. (5))
  const int head = blockIdx.x % h, grp = blockIdx.x / h, s = blockIdx.y;
  const int bpg = n_blocks / groups, b0 = grp * bpg;
  const int n = seq_lens[s];
  const int active = min(n_splits, (n + chunk - 1) / chunk);
  const int tid = threadIdx.x;
  for (int bb = 0; bb < bpg; ++bb) {
    const int b = b0 + bb;
    const size_t unit0 = ((size_t)s * n_blocks + b) * n_splits;
    float m_star = kNegBig;
    for (int k = 0; k < active; ++k) m_star = fmaxf(m_star, part_ml[((unit0 + k) * h + head) * 2]);
    float L = 0.f;
    for (int k = 0; k < active; ++k) {
      const float* ml = part_ml + ((unit0 + k) * h + head) * 2;
      L += exp2f(ml[0] - m_star) * ml[1];
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    for (int c = tid; c < d_cb; c += 256) {
      float z = 0.f;
      for (int k = 0; k < active; ++k) {
        const float w = exp2f(part_ml[((unit0 + k) * h + head) * 2] - m_star);
        z += w * part_z[((unit0 + k) * h + head) * d_cb + c];
      }
      zs[bb * d_cb + c] = z * inv;
    }
    if (tid == 0 && lse) lse[((size_t)s * n_blocks + b) * h + head] = L > 0.f ? (m_star + log2f(L)) * kLn2 : -INFINITY;
  }
  __syncthreads();
  const int d_cg = bpg * d_cb;
  const size_t ld = (size_t)h * d_h;
  for (int j = tid; j < d_h; j += 256) {
    float acc = 0.f;
    for (int r = 0; r < d_cg; ++r)
      acc += zs[r] * load_f32(w_uv, ((size_t)b0 * d_cb + r) * ld + (size_t)head * d_h + j);
    const size_t o = ((size_t)s * h * groups + blockIdx.x) * d_h + j;
    store_f32(out, o, acc * out_scale * (gate ? load_f32(gate, o) : 1.f));   // gate: Appendix E, O^attn = Attention . G
  }
}

int launch_merge_upproj_generic(const DecodeArgs& a) {
  dim3 grid(a.h * a.groups, a.batch);
  const size_t lds = (size_t)a.n_blocks / a.groups * a.d_cb * sizeof(float);
#define MLRA_MERGE(T, TO)                                                                                       \
  merge_upproj_generic_kernel<T, TO><<<grid, 256, lds, a.stream>>>(                                             \
      a.part_z, a.part_ml, a.seq_lens, (const T*)a.w_uv, (TO*)a.out, a.lse, a.h, a.d_h, a.n_blocks, a.d_cb,     \
      a.plan.n_splits, a.plan.chunk_tokens, a.out_scale, a.groups, (const T*)a.gate)
  if (a.dtype == MLRA_BF16 && a.out_dtype == MLRA_BF16) MLRA_MERGE(bf16_t, bf16_t);
  else if (a.dtype == MLRA_BF16) MLRA_MERGE(bf16_t, float);
  else if (a.out_dtype == MLRA_BF16) MLRA_MERGE(float, bf16_t);
  else MLRA_MERGE(float, float);
#undef MLRA_MERGE
  return check_launch();
}

// ------------------------------------------------------------------------------------------------
// GQA decode, generic form (Appendix C, MQA/GQA): one workgroup per (chunk, KV head x query-head
// group, sequence); K and V tiles of TT tokens in LDS as fp32.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gqa_generic_kernel(
    const T* __restrict__ k_pool, const T* __restrict__ v_pool, const int32_t* __restrict__ page_table,
    const int32_t* __restrict__ seq_lens, int page_size, int max_pages, int h, int g, int d_h,
    const T* __restrict__ q, float scale_log2, float* __restrict__ part_o, float* __restrict__ part_ml,
    int n_splits, int chunk, int HG, int TT) {
  extern __shared__ float smem[];
  const int DP = d_h + 1;
  float* qs = smem;               // [HG][d_h]
  float* kt = qs + HG * d_h;      // [TT][DP]
  float* vt = kt + TT * DP;       // [TT][DP]
  float* ps = vt + TT * DP;       // [HG][TT]
  float* zs = ps + HG * TT;       // [HG][d_h]
  float* ms = zs + HG * d_h;
  float* ls = ms + HG;
  float* al = ls + HG;

  const int r = h / g;
  const int n_sub = (r + HG - 1) / HG;
  const int j = blockIdx.y / n_sub, sub = blockIdx.y % n_sub;
  const int split = blockIdx.x, s = blockIdx.z;
  const int n = seq_lens[s];
  const int t0 = split * chunk;
  if (t0 >= n) return;
  const int t1 = min(n, t0 + chunk);
  const int head0 = j * r + sub * HG;
  const int nh = min(HG, r - sub * HG);
  const int tid = threadIdx.x;

  for (int idx = tid; idx < nh * d_h; idx += 256)
    qs[idx] = load_f32(q, ((size_t)s * h + head0 + idx / d_h) * d_h + idx % d_h);
  for (int idx = tid; idx < HG * d_h; idx += 256) zs[idx] = 0.f;
  if (tid < HG) { ms[tid] = kNegBig; ls[tid] = 0.f; al[tid] = 1.f; }
  __syncthreads();

  for (int tb = t0; tb < t1; tb += TT) {
    for (int idx = tid; idx < TT * d_h; idx += 256) {
      const int t = idx / d_h, k = idx % d_h;
      const int tok = tb + t;
      float kv = 0.f, vv = 0.f;
      if (tok < t1) {
        const int page = page_table[(size_t)s * max_pages + tok / page_size];
        const size_t off = (((size_t)page * g + j) * page_size + tok % page_size) * d_h + k;
        kv = load_f32(k_pool, off);
        vv = load_f32(v_pool, off);
      }
      kt[t * DP + k] = kv;
      vt[t * DP + k] = vv;
    }
    __syncthreads();
    for (int idx = tid; idx < nh * TT; idx += 256) {
      const int hh = idx / TT, t = idx % TT;
      float acc = 0.f;
      for (int k = 0; k < d_h; ++k) acc += qs[hh * d_h + k] * kt[t * DP + k];
      ps[hh * TT + t] = (tb + t < t1) ? acc * scale_log2 : -INFINITY;
    }
    __syncthreads();
    {
      const int wave = tid / 64, lane = tid % 64;
      for (int hh = wave; hh < nh; hh += 4) {
        const float sc = lane < TT ? ps[hh * TT + lane] : -INFINITY;
        const float m_old = ms[hh];
        const float m_new = fmaxf(m_old, wave_max(sc));
        const float p = exp2f(sc - m_new);
        const float sum = wave_sum(p);
        if (lane < TT) ps[hh * TT + lane] = p;
        if (lane == 0) {
          const float a = exp2f(m_old - m_new);
          al[hh] = a;
          ms[hh] = m_new;
          ls[hh] = ls[hh] * a + sum;
        }
      }
    }
    __syncthreads();
    for (int idx = tid; idx < nh * d_h; idx += 256) {
      const int hh = idx / d_h, c = idx % d_h;
      float acc = zs[idx] * al[hh];
      for (int t = 0; t < TT; ++t) acc += ps[hh * TT + t] * vt[t * DP + c];
      zs[idx] = acc;
    }
    __syncthreads();
  }
  const size_t unit = (size_t)s * n_splits + split;
  for (int idx = tid; idx < nh * d_h; idx += 256)
    part_o[(unit * h + head0 + idx / d_h) * d_h + idx % d_h] = zs[idx];
  if (tid < nh) {
    part_ml[(unit * h + head0 + tid) * 2 + 0] = ms[tid];
    part_ml[(unit * h + head0 + tid) * 2 + 1] = ls[tid];
  }
}

int launch_gqa_generic(const GqaArgs& a) {
  const int r = a.h / a.g;
  const int HG = r < 16 ? r : 16;
  int TT = 64;
  auto lds_bytes = [&](int tt) {
    return (size_t)(HG * a.d_h + 2 * tt * (a.d_h + 1) + HG * tt + HG * a.d_h + 3 * HG) * 4;
  };
  while (TT > 1 && lds_bytes(TT) > 64 * 1024) TT >>= 1;
  if (lds_bytes(TT) > 64 * 1024) return MLRA_ERR_SHAPE;
  const int n_sub = (r + HG - 1) / HG;
  dim3 grid(a.plan.n_splits, a.g * n_sub, a.batch);
  const float scale_log2 = softmax_scale_log2(a.softmax_scale);
  if (a.dtype == MLRA_BF16)
    gqa_generic_kernel<bf16_t><<<grid, 256, lds_bytes(TT), a.stream>>>(
        (const bf16_t*)a.k_pool, (const bf16_t*)a.v_pool, a.page_table, a.seq_lens, a.page_size, a.max_pages, a.h,
        a.g, a.d_h, (const bf16_t*)a.q, scale_log2, a.part_o, a.part_ml, a.plan.n_splits, a.plan.chunk_tokens, HG, TT);
  else
    gqa_generic_kernel<float><<<grid, 256, lds_bytes(TT), a.stream>>>(
        (const float*)a.k_pool, (const float*)a.v_pool, a.page_table, a.seq_lens, a.page_size, a.max_pages, a.h,
        a.g, a.d_h, (const float*)a.q, scale_log2, a.part_o, a.part_ml, a.plan.n_splits, a.plan.chunk_tokens, HG, TT);
  return check_launch();
}

template <typename TO>
__global__ __launch_bounds__(256) void gqa_merge_kernel(const float* __restrict__ part_o,
                                                        const float* __restrict__ part_ml,
                                                        const int32_t* __restrict__ seq_lens, TO* __restrict__ out,
                                                        int h, int d_h, int n_splits, int chunk) {
  const int head = blockIdx.x, s = blockIdx.y;
  const int n = seq_lens[s];
  const int active = min(n_splits, (n + chunk - 1) / chunk);
  const size_t unit0 = (size_t)s * n_splits;
  float m_star = kNegBig;
  for (int k = 0; k < active; ++k) m_star = fmaxf(m_star, part_ml[((unit0 + k) * h + head) * 2]);
  float L = 0.f;
  for (int k = 0; k < active; ++k) {
    const float* ml = part_ml + ((unit0 + k) * h + head) * 2;
    L += exp2f(ml[0] - m_star) * ml[1];
  }
  const float inv = L > 0.f ? 1.f / L : 0.f;
  for (int c = threadIdx.x; c < d_h; c += 256) {
    float z = 0.f;
    for (int k = 0; k < active; ++k)
      z += exp2f(part_ml[((unit0 + k) * h + head) * 2] - m_star) * part_o[((unit0 + k) * h + head) * d_h + c];
    store_f32(out, ((size_t)s * h + head) * d_h + c, z * inv);
  }
}

int launch_gqa_merge(const GqaArgs& a) {
  dim3 grid(a.h, a.batch);
  if (a.out_dtype == MLRA_BF16)
    gqa_merge_kernel<bf16_t><<<grid, 256, 0, a.stream>>>(a.part_o, a.part_ml, a.seq_lens, (bf16_t*)a.out, a.h, a.d_h,
                                                         a.plan.n_splits, a.plan.chunk_tokens);
  else
    gqa_merge_kernel<float><<<grid, 256, 0, a.stream>>>(a.part_o, a.part_ml, a.seq_lens, (float*)a.out, a.h, a.d_h,
                                                        a.plan.n_splits, a.plan.chunk_tokens);
  return check_launch();
}

}  // namespace mlra
